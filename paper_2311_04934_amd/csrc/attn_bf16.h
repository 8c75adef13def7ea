// Declarations shared by the two bf16 attention kernels (register-staged: attn_bf16.hip; DMA-staged:
// attn_bf16_wide.hip; both 32 query rows per wave) and their launcher.
#pragma once

#include "common.h"
#include "kv_seg.h"

namespace pc {
namespace attn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int KT = 64;          // keys per LDS tile
constexpr int RW = 32;          // query rows per wave
constexpr int kPosInf = 0x7fffffff;
// Online softmax keeps a per-query reference maximum (log2 domain).  It is only moved when a
// new score exceeds it by more than kMaxSlack, so that the accumulators need rescaling only
// rarely; probabilities then range up to 2^kMaxSlack, which bf16 and fp32 hold without loss.
constexpr float kMaxSlack = 8.0f;

// Kernel argument of both bf16 kernels.  The fields a workgroup needs first come first, and the first prompt is
// repeated ahead of the table (seq0), so that a call with one prompt finds its work unit with the first look at
// the arguments instead of a second, dependent one.
struct AttnParams {
    int Hq, Hkv, G;
    int n_splits;
    int rb_max;              // row blocks per (prompt, kv head)
    int n_groups;            // n_seqs * n_splits * Hkv
    int n_seqs;
    AttnSeq seq0;            // = batch.seq[0]
    int q_rotated;           // Q comes rotated and scaled (log2(e)/sqrt(D)) already: its bf16 values are the operand
    int max_pos;
    int total_q;
    float q_scale;           // log2(e) / sqrt(D)
    const uint16_t *q;       // [total_q][Hq][D] bf16 bits
    const int32_t *q_pos;
    const uint16_t *k;       // [total_kv][Hkv][D]
    const uint16_t *v;
    const int32_t *kv_pos;
    uint16_t *out;           // [total_q][Hq][D]
    // Un-normalised partial O (bf16) and (m, l) of every KV split: [n_splits][total_q][Hq] rows in the register-staged
    // kernel, [n_splits][Hq][total_q] rows in the DMA-staged one.
    uint16_t *part_o;
    float2 *part_ml;
    const float2 *rope;      // [max_pos][D/2]
    const float2 *rope_t;    // [D/2][max_pos]
    const float *alibi;      // [Hq] slopes of the linear bias, or nullptr: rotation
    AttnBatch batch;
};


__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// all-reduce over the 64 lanes of a wave with DPP row rotations and the row/half swaps of gfx950
#define PC_WAVE_ALLREDUCE(NAME, T, OP)                                                                   \
    __device__ __forceinline__ T NAME(T x)                                                               \
    {                                                                                                    \
        x = OP(x, (T)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x128, 0xf, 0xf, false)); /* ror 8 */  \
        x = OP(x, (T)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x124, 0xf, 0xf, false)); /* ror 4 */  \
        x = OP(x, (T)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x122, 0xf, 0xf, false)); /* ror 2 */  \
        x = OP(x, (T)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x121, 0xf, 0xf, false)); /* ror 1 */  \
        const u32x2 a = __builtin_amdgcn_permlane16_swap((unsigned)x, (unsigned)x, false, false);        \
        x = OP((T)a[0], (T)a[1]);                                                                        \
        const u32x2 b = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);        \
        return OP((T)b[0], (T)b[1]);                                                                     \
    }
__device__ __forceinline__ int pc_imin(int a, int b) { return a < b ? a : b; }
__device__ __forceinline__ int pc_imax(int a, int b) { return a > b ? a : b; }
PC_WAVE_ALLREDUCE(wave_min_i32, int, pc_imin)
PC_WAVE_ALLREDUCE(wave_max_i32, int, pc_imax)
#undef PC_WAVE_ALLREDUCE

// max / sum over the two halves of the wave (lane l and lane l^32 end up with the same value)
__device__ __forceinline__ float max_across_halves(float x)
{
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float x)
{
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

}  // namespace attn

// DMA-staged kernel (attn_bf16_wide.hip): D = 128, 8 row tiles per workgroup, 1 row tile per wave.
// tab != nullptr: K/V and positions are read through the segment table (p.k, p.v, p.kv_pos unused).
int launch_attn_bf16_wide(pc_ctx *ctx, attn::AttnParams &p, int n_blocks, hipStream_t stream,
                          const KvSegTable *tab = nullptr);
constexpr int kWideRowTilesPerWg = 8;
constexpr int kWideMinRowTiles = 1;     // measured: the DMA-staged kernel is ~2x faster even with 1-3 row tiles per kv head (its other waves stage)

}  // namespace pc
