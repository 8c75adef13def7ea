// RoPE at arbitrary position IDs, and the append of the uncached tokens' own K/V.
//
// Prompt modules are encoded at the position IDs their schema fixes, which do not
// start at zero and are not contiguous across a prompt (Sec. 3.3 of the paper);
// the rotation is therefore looked up by position ID in a table (Sec. 4.2).  The
// table holds (cos, sin) of pos * base^(-2i/d), computed in fp64 on the host and
// rounded once to fp32, so the angle carries no fp32 range-reduction error even
// at positions in the tens of thousands.  Pairing is half-split: element i rotates
// with element i + d/2.
#include "common.h"

namespace pc {
namespace {

template <typename T>
struct Elem;
template <>
struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float x) { *p = x; }
};
template <>
struct Elem<uint16_t> {  // bf16 bits
    static __device__ __forceinline__ float load(const uint16_t *p) { return __uint_as_float((uint32_t)*p << 16); }
    static __device__ __forceinline__ void store(uint16_t *p, float x) { *p = __builtin_bit_cast(uint16_t, (__bf16)x); }
};

__device__ __forceinline__ int clamp_pos(int pos, int max_pos) { return pos < 0 ? 0 : (pos >= max_pos ? max_pos - 1 : pos); }

// One thread per rotation pair.
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T *x, int n_tokens, int n_heads, int d, const int32_t *pos,
                                                   const float2 *table, int max_pos)
{
    const int half = d >> 1;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const long total = (long)n_tokens * n_heads * half;
    if (idx >= total) return;
    const int i = (int)(idx % half);
    const long th = idx / half;  // token * n_heads + head
    const int t = (int)(th / n_heads);
    const float2 cs = table[(size_t)clamp_pos(pos[t], max_pos) * half + i];
    T *row = x + (size_t)th * d;
    const float lo = Elem<T>::load(row + i), hi = Elem<T>::load(row + i + half);
    Elem<T>::store(row + i, lo * cs.x - hi * cs.y);
    Elem<T>::store(row + i + half, hi * cs.x + lo * cs.y);
}

// One workgroup per appended row: rotate K_new at the row's position ID into the tail of
// the assembled K, copy V_new, write the position ID.
template <typename T>
__global__ __launch_bounds__(256) void append_kernel(const AppendArgs a, const T *k_new, const T *v_new,
                                                     const int32_t *q_pos, T *asm_k, T *asm_v, int32_t *asm_pos,
                                                     int n_kv_heads, int d, const float2 *table, int max_pos)
{
    // which prompt does this row belong to (uniform scan over at most kMaxAppendSegs entries)
    int r = blockIdx.x, s = 0;
    while (s < a.n_segs && r >= a.seg[s].n) {
        r -= a.seg[s].n;
        ++s;
    }
    if (s >= a.n_segs) return;
    const int src = a.seg[s].q_begin + r;
    const int dst = a.seg[s].dst_row + r;
    const int half = d >> 1;
    const int row_elems = n_kv_heads * d;
    const int p = q_pos[src];
    const float2 *trow = table + (size_t)clamp_pos(p, max_pos) * half;
    const T *ks = k_new + (size_t)src * row_elems;
    const T *vs = v_new + (size_t)src * row_elems;
    T *kd = asm_k + (size_t)dst * row_elems;
    T *vd = asm_v + (size_t)dst * row_elems;
    for (int e = threadIdx.x; e < n_kv_heads * half; e += 256) {
        const int h = e / half, i = e % half;
        const float2 cs = trow[i];
        const float lo = Elem<T>::load(ks + h * d + i), hi = Elem<T>::load(ks + h * d + i + half);
        Elem<T>::store(kd + h * d + i, lo * cs.x - hi * cs.y);
        Elem<T>::store(kd + h * d + i + half, hi * cs.x + lo * cs.y);
    }
    for (int e = threadIdx.x; e < row_elems; e += 256) vd[e] = vs[e];
    if (threadIdx.x == 0) asm_pos[dst] = p;
}

}  // namespace

int launch_rope(pc_ctx *ctx, void *x, int n_tokens, int n_heads, const int32_t *pos, hipStream_t stream)
{
    const int head_dim = ctx->cfg.head_dim, max_pos = ctx->cfg.max_pos;
    const float2 *table = ctx->rope_table;
    const long total = (long)n_tokens * n_heads * (head_dim / 2);
    if (total <= 0) return PC_OK;
    const int blocks = (int)((total + 255) / 256);
    if (ctx->cfg.dtype == PC_F32)
        return launch_kernel(ctx, kProfRope, rope_kernel<float>, dim3(blocks), dim3(256), 0, stream,
                             static_cast<float *>(x), n_tokens, n_heads, head_dim, pos, table, max_pos);
    return launch_kernel(ctx, kProfRope, rope_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream,
                         static_cast<uint16_t *>(x), n_tokens, n_heads, head_dim, pos, table, max_pos);
}

int launch_append(pc_ctx *ctx, const AppendArgs &args, const void *k_new, const void *v_new, const int32_t *q_pos,
                  void *asm_k, void *asm_v, int32_t *asm_pos, hipStream_t stream)
{
    if (args.total_rows <= 0) return PC_OK;
    const int n_kv_heads = ctx->cfg.n_kv_heads, head_dim = ctx->cfg.head_dim, max_pos = ctx->cfg.max_pos;
    const float2 *table = ctx->rope_table;
    if (ctx->cfg.dtype == PC_F32)
        return launch_kernel(ctx, kProfAppend, append_kernel<float>, dim3(args.total_rows), dim3(256), 0, stream, args,
                             static_cast<const float *>(k_new), static_cast<const float *>(v_new), q_pos,
                             static_cast<float *>(asm_k), static_cast<float *>(asm_v), asm_pos, n_kv_heads, head_dim,
                             table, max_pos);
    return launch_kernel(ctx, kProfAppend, append_kernel<uint16_t>, dim3(args.total_rows), dim3(256), 0, stream, args,
                         static_cast<const uint16_t *>(k_new), static_cast<const uint16_t *>(v_new), q_pos,
                         static_cast<uint16_t *>(asm_k), static_cast<uint16_t *>(asm_v), asm_pos, n_kv_heads, head_dim,
                         table, max_pos);
}

}  // namespace pc
