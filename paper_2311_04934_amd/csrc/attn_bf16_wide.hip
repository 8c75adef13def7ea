// Uncached-token prefill attention over the assembled KV (Sec. 3.4 of the paper), bf16 MFMA,
// "wide" variant for head_dim 128: 4 wavefronts per workgroup, 64 query rows per wavefront.
//
// Same contract and the same S^T = K.Q^T / O^T += V^T.P^T formulation as the narrow kernel
// (attn_bf16.hip); what differs is how the work is fed:
//
//   rows      a wave owns TWO 32-query row tiles (a, b).  Every K and V fragment read from LDS
//             feeds two MFMAs, which halves the LDS traffic per FLOP (the narrow kernel is
//             bound by LDS bandwidth at head_dim 128).
//   staging   K, V and position IDs of a 64-key tile go from global memory straight into LDS
//             (global_load_lds, 16 bytes per lane): no registers, no LDS-write instructions.
//             Four tile buffers; the loads of tile T+3 are issued while tile T is computed.
//             Rows are stored unpadded with their 16-byte chunks XOR-swizzled by the key index
//             so that both the K reads (one key per lane) and the transposing V reads are
//             bank-conflict free.
//   V         stays row-major [key][d] in LDS; the MFMA A operand V^T is fetched with
//             ds_read_b64_tr_b16, which hands every lane four keys of one d column.
//   pipeline  one wave per SIMD, so matrix and vector work of the SAME wave are interleaved:
//               phase 1(i):  softmax of tile a, sub-tile i   ||  P.V MFMAs of sub-tile i-1 (a and b)
//               phase 2(i):  softmax of tile b, sub-tile i   ||  K.Q MFMAs of sub-tile i+1 (a and b)
//             each phase is one straight-line block of 16 MFMAs and ~100 vector instructions.
//             Rescaling O when a running maximum moved is deferred to the start of the next
//             phase 1 and skipped when no lane needs it.
//   epilogue  O^T goes through LDS so that partial results / outputs are written as whole rows.
#include <stdlib.h>

#include "attn_bf16.h"

namespace pc {
namespace {

using namespace attn;

constexpr int D = 128;
constexpr int KB = D / 16;       // MFMA k-blocks over the head dim (K.Q)
constexpr int DB = D / 32;       // 32-row blocks of O^T
constexpr int NBUF = 4;
constexpr int ROW_BYTES = D * 2;                 // one K or V row of one head
constexpr int TILE_BYTES = KT * ROW_BYTES;       // 16 KiB
constexpr int LDS_K = 0;
constexpr int LDS_V = NBUF * TILE_BYTES;         // 64 KiB
constexpr int LDS_POS = 2 * NBUF * TILE_BYTES;   // 128 KiB
constexpr int LDS_MAIN = LDS_POS + NBUF * KT * 4;
constexpr int EPI_STRIDE = D * 4 + 16;           // fp32 row of O plus a 16-byte pad
constexpr int LDS_EPI = 256 * EPI_STRIDE;        // 256 query rows per workgroup
constexpr int LDS_TOTAL = LDS_MAIN > LDS_EPI ? LDS_MAIN : LDS_EPI;

typedef __attribute__((address_space(3))) uint8_t lds_u8;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// s_waitcnt that only waits for the vector-memory counter to drop to n (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "don't wait").
#define PC_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// Asynchronous global -> LDS copy of 16 (or 4) bytes per lane: lane l's data lands at
// lds_addr + 16*l (4*l).  Issued as inline assembly so that the compiler does not make every
// later LDS read wait for it; completion is awaited explicitly with PC_WAIT_VMCNT before the
// workgroup barrier that publishes a tile.
__device__ __forceinline__ void dma_b128(const void *gsrc, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gsrc) : "memory");
}
__device__ __forceinline__ void dma_b32(const void *gsrc, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(gsrc) : "memory");
}

struct QTile {        // one 32-query row tile of a wave
    bool valid;       // this lane's query exists
    int head;
    int qi;           // query index inside the prompt
    int qpos;         // its position ID (+inf when the lane has no query)
};

template <int NQT, int NW>
__global__ __launch_bounds__(NW * 64) void attn_bf16_dma_kernel(const AttnParams p)
{
    static_assert(NQT * NW == kWideRowTilesPerWg, "a workgroup covers 8 row tiles");
    constexpr int GRP_PER_WAVE = 16 / NW;                // 1-KiB (4-row) groups of a tile each wave copies, per tensor
    constexpr int DMA_PER_TILE = 2 * GRP_PER_WAVE + 1;   // loads a wave issues per tile (K, V, positions)

    extern __shared__ __align__(16) uint8_t smem[];
    lds_u8 *lds = (lds_u8 *)smem;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;
    const int hh = lane >> 5;

    // ---- work unit (same XCD-aware enumeration as the narrow kernel)
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int g = (slot / p.rb_max) * 8 + xcd;
    const int rb = slot % p.rb_max;
    if (g >= p.n_groups) return;
    const int split = g % p.n_splits;
    const int seq_i = (g / p.n_splits) % p.batch.n_seqs;
    const int kvh = g / (p.n_splits * p.batch.n_seqs);
    const AttnSeq seq = p.batch.seq[seq_i];

    const int tiles_q = (seq.n_q + RW - 1) / RW;
    const int row_tiles = p.G * tiles_q;
    if (rb * kWideRowTilesPerWg >= row_tiles) return;

    const int share = (((seq.n_kv + p.n_splits - 1) / p.n_splits) + 31) & ~31;
    const int k_begin = split * share < seq.n_kv ? split * share : seq.n_kv;
    const int k_end = k_begin + share < seq.n_kv ? k_begin + share : seq.n_kv;
    const int n_tiles = (k_end - k_begin + KT - 1) / KT;

    // ---- this wave's two row tiles
    QTile qt[NQT];
#pragma unroll
    for (int x = 0; x < NQT; ++x) {
        const int rt = rb * kWideRowTilesPerWg + wave * NQT + x;
        const bool act = rt < row_tiles;
        const int g_head = act ? rt / tiles_q : 0;
        const int tq = act ? rt % tiles_q : 0;
        qt[x].head = kvh * p.G + g_head;
        qt[x].qi = tq * RW + col;
        qt[x].valid = act && qt[x].qi < seq.n_q;
        qt[x].qpos = qt[x].valid ? p.q_pos[seq.q_begin + qt[x].qi] : kPosInf;
    }

    const size_t kv_row_stride = (size_t)p.Hkv * D;  // elements
    const uint16_t *k_base = p.k + (size_t)seq.kv_begin * kv_row_stride + (size_t)kvh * D;
    const uint16_t *v_base = p.v + (size_t)seq.kv_begin * kv_row_stride + (size_t)kvh * D;
    const int32_t *pos_base = p.kv_pos + seq.kv_begin;
    const int last_row = k_end - 1;

    // ---- global -> LDS, asynchronously.  One wave instruction fills 1 KiB = 4 rows; LDS slot
    // (row r, 16-byte chunk c) receives global chunk c ^ swz(r).  Rows past the split's end are
    // read from its last row (finite values; they are masked by index in the softmax).
    // Every wave issues exactly 9 loads per tile.
    const int st_row = lane >> 4;          // row inside a 4-row group
    const int st_chunk = lane & 15;
    const uint32_t row_bytes_g = (uint32_t)kv_row_stride * 2u;   // bytes between consecutive keys in global memory
    const uint8_t *k_bytes = reinterpret_cast<const uint8_t *>(k_base);
    const uint8_t *v_bytes = reinterpret_cast<const uint8_t *>(v_base);
    uint32_t dma_r[GRP_PER_WAVE], dma_ck[GRP_PER_WAVE], dma_cv[GRP_PER_WAVE];
#pragma unroll
    for (int j = 0; j < GRP_PER_WAVE; ++j) {
        const int r = (j * NW + wave) * 4 + st_row;                // row of the tile this lane fetches in step j
        dma_r[j] = (uint32_t)r;
        dma_ck[j] = (uint32_t)((st_chunk ^ (r & 15)) << 4);       // byte offset of the chunk inside the row
        dma_cv[j] = (uint32_t)((st_chunk ^ ((r & 7) << 1)) << 4);
    }
    auto issue_tile = [&](int t) {
        const int buf = t & (NBUF - 1);
        const uint32_t row0 = (uint32_t)(k_begin + t * KT);
        const uint32_t dst0 = __builtin_amdgcn_readfirstlane(lds_base + buf * TILE_BYTES + wave * 1024);
#pragma unroll
        for (int j = 0; j < GRP_PER_WAVE; ++j) {
            uint32_t grow = row0 + dma_r[j];
            grow = grow < (uint32_t)last_row ? grow : (uint32_t)last_row;
            const uint32_t off = grow * row_bytes_g;               // < 4 GiB, checked by the launcher
            dma_b128(k_bytes + off + dma_ck[j], dst0 + LDS_K + j * NW * 1024);
            dma_b128(v_bytes + off + dma_cv[j], dst0 + LDS_V + j * NW * 1024);
        }
        uint32_t prow = row0 + (uint32_t)lane;
        prow = prow < (uint32_t)last_row ? prow : (uint32_t)last_row;
        dma_b32(pos_base + prow, __builtin_amdgcn_readfirstlane(lds_base + LDS_POS + buf * KT * 4));
    };

    // ---- prologue: Q of both row tiles, rotated at the queries' position IDs, scaled, bf16
    bf16x8 qf[NQT][KB];
#pragma unroll
    for (int x = 0; x < NQT; ++x) {
        const int q_row = seq.q_begin + (qt[x].valid ? qt[x].qi : 0);
        const uint16_t *qrow = p.q + ((size_t)q_row * p.Hq + qt[x].head) * D;
        int tpos = qt[x].qpos;
        tpos = tpos < 0 ? 0 : (tpos >= p.max_pos ? p.max_pos - 1 : tpos);
        const float2 *trow = p.rope + (size_t)tpos * (D / 2);
#pragma unroll
        for (int kb = 0; kb < KB / 2; ++kb) {
            const int d0 = kb * 16 + hh * 8;
            u32x4 lo = *reinterpret_cast<const u32x4 *>(qrow + d0);
            u32x4 hi = *reinterpret_cast<const u32x4 *>(qrow + d0 + D / 2);
            bf16x8 olo, ohi;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint32_t wl = lo[e >> 1], wh = hi[e >> 1];
                float xl = bf16_bits_to_f32((e & 1) ? (wl >> 16) : (wl & 0xffffu));
                float xh = bf16_bits_to_f32((e & 1) ? (wh >> 16) : (wh & 0xffffu));
                float2 cs = trow[d0 + e];
                olo[e] = (__bf16)((xl * cs.x - xh * cs.y) * p.q_scale);
                ohi[e] = (__bf16)((xh * cs.x + xl * cs.y) * p.q_scale);
            }
            qf[x][kb] = olo;
            qf[x][kb + KB / 2] = ohi;
        }
    }
    // smallest query position in the wave: a key tile whose largest position exceeds it needs the mask
    int min_qpos = qt[0].qpos;
#pragma unroll
    for (int x = 1; x < NQT; ++x) min_qpos = pc_imin(min_qpos, qt[x].qpos);
    const int wave_min_qpos = wave_min_i32(min_qpos);

    // first three tiles on their way (after the Q loads, so that waiting for Q does not wait for them)
    if (n_tiles > 0) issue_tile(0);
    if (n_tiles > 1) issue_tile(1);
    if (n_tiles > 2) issue_tile(2);

    // ---- per-lane LDS offsets of the MFMA operand fragments
    // K (A operand of K.Q): key = col of the sub-tile, chunk 2*kb+hh, swizzled by key & 15
    int koff[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) koff[kb] = col * ROW_BYTES + (((2 * kb + hh) ^ (col & 15)) << 4);
    // V (A operand of V^T.P via the transposing read): lane (16-lane group gq, member jq) points at
    // key 4*(gq>>1) + (jq>>2) (+ 16*j + 8*u per instruction), d = 32*b + 16*(gq&1) + 4*(jq&3)
    int voff[DB];
    {
        const int gq = lane >> 4, jq = lane & 15;
        const int key_lo = 4 * (gq >> 1) + (jq >> 2);            // = key & 7
        const int swz = key_lo << 1;
#pragma unroll
        for (int b = 0; b < DB; ++b) {
            const int chunk = 4 * b + 2 * (gq & 1) + ((jq & 3) >> 1);
            voff[b] = key_lo * ROW_BYTES + ((chunk ^ swz) << 4) + 8 * (jq & 1);
        }
    }

    // ---- state
    f32x16 o_acc[NQT][DB];
    float m_run[NQT], l_run[NQT], alpha[NQT];   // running max / sum; alpha = pending rescale of O
    bf16x8 pf[2][NQT][2];          // [sub-tile parity][row tile][16-key half]
    f32x16 sc[2][NQT];             // [sub-tile parity][row tile] scores
#pragma unroll
    for (int x = 0; x < NQT; ++x) {
        m_run[x] = -INFINITY;
        l_run[x] = 0.f;
        alpha[x] = 1.f;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) o_acc[x][b][i] = 0.f;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[a][x][j][e] = (__bf16)0.f;
    }

    // K.Q for the wave's row tiles on one 32-key sub-tile: every K fragment is read once
    auto qk = [&](int buf, int sub, f32x16 (&s)[NQT]) {
        const lds_u8 *base = lds + LDS_K + buf * TILE_BYTES + sub * 32 * ROW_BYTES;
#pragma unroll
        for (int x = 0; x < NQT; ++x)
#pragma unroll
            for (int i = 0; i < 16; ++i) s[x][i] = 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const u32x4 raw = *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(base + koff[kb]);
            const bf16x8 kf = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
            for (int x = 0; x < NQT; ++x) s[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[x][kb], s[x], 0, 0, 0);
        }
    };

    // O^T += V^T.P^T for the wave's row tiles on one sub-tile: every V fragment is read once
    auto pv = [&](int buf, int sub, const bf16x8 (&pp)[NQT][2]) {
        const lds_u8 *base = lds + LDS_V + buf * TILE_BYTES + sub * 32 * ROW_BYTES;
#pragma unroll
        for (int b = 0; b < DB; ++b) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const lds_u8 *a0 = base + voff[b] + (16 * j) * ROW_BYTES;
                const s16x4 t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a0);
                const s16x4 t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(a0 + 8 * ROW_BYTES));
                const s16x8 t = __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 vf = __builtin_bit_cast(bf16x8, t);
#pragma unroll
                for (int x = 0; x < NQT; ++x)
                    o_acc[x][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pp[x][j], o_acc[x][b], 0, 0, 0);
            }
        }
    };

    // online softmax of one score tile (row tile x); O is NOT rescaled here (see rescale())
    auto softmax = [&](bool masked, f32x16 &s, int x, int buf, int sub, int n_valid, bf16x8 (&pout)[2]) {
        if (masked) {
            const lds_u8 *pp = lds + LDS_POS + buf * KT * 4;
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int key0 = sub * 32 + 8 * i4 + 4 * hh;
                const u32x4 kp = *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(pp + key0 * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((int)kp[e] > qt[x].qpos || key0 + e >= n_valid) s[i4 * 4 + e] = -INFINITY;
            }
        }
        float mx = s[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i]);
        mx = max_across_halves(mx);
        const float m_new = mx > m_run[x] + kMaxSlack ? mx : m_run[x];
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float a = __builtin_amdgcn_exp2f(m_run[x] - m_use);
        m_run[x] = m_new;
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float pe = __builtin_amdgcn_exp2f(s[i] - m_use);
            psum += pe;
            pout[i >> 3][i & 7] = (__bf16)pe;
        }
        l_run[x] = l_run[x] * a + psum;
        alpha[x] = a;
    };

    auto rescale = [&]() {
        bool need = false;
#pragma unroll
        for (int x = 0; x < NQT; ++x) need |= alpha[x] != 1.f;
        if (__any(need)) {
#pragma unroll
            for (int x = 0; x < NQT; ++x)
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o_acc[x][b][i] *= alpha[x];
        }
    };

    // does tile t (already visible in LDS) need the per-element mask for this wave?
    auto tile_needs_mask = [&](int t) -> bool {
        const int buf = t & (NBUF - 1);
        const int n_valid = k_end - (k_begin + t * KT);
        const int pv_ = *reinterpret_cast<const __attribute__((address_space(3))) int *>(lds + LDS_POS + buf * KT * 4 + lane * 4);
        const int tmax = wave_max_i32(pv_);
        return __builtin_amdgcn_readfirstlane(tmax > wave_min_qpos || n_valid < KT);
    };

    // ---- main loop
    if (n_tiles > 0) {
        // tile 0 visible
        if (n_tiles > 2) PC_WAIT_VMCNT(2 * DMA_PER_TILE);
        else if (n_tiles > 1) PC_WAIT_VMCNT(DMA_PER_TILE);
        else PC_WAIT_VMCNT(0);
        __syncthreads();
        bool mask_cur = tile_needs_mask(0);
        qk(0, 0, sc[0]);

        for (int t = 0; t < n_tiles; ++t) {
            const int buf = t & (NBUF - 1);
            const int n_valid = k_end - (k_begin + t * KT);   // real keys in this tile (may exceed 64)
            const bool has_next = t + 1 < n_tiles;
            // previous sub-tile (for P.V): sub 1 of tile t-1; for t == 0 any finite data times P = 0
            const int pbuf = t > 0 ? (t - 1) & (NBUF - 1) : buf;
            const int psub = t > 0 ? 1 : 0;

            // ===== sub-tile 0 of tile t: scores in sc[0]
            rescale();
            pv(pbuf, psub, pf[1]);
#pragma unroll
            for (int x = 0; x < NQT; ++x) softmax(mask_cur, sc[0][x], x, buf, 0, n_valid, pf[0][x]);
            qk(buf, 1, sc[1]);

            // make tile t+1 visible; its loads were issued two tiles ago.  Loads of tile t+2 may stay in flight.
            if (t + 2 < n_tiles) PC_WAIT_VMCNT(DMA_PER_TILE);
            else PC_WAIT_VMCNT(0);
            __syncthreads();
            if (t + 3 < n_tiles) issue_tile(t + 3);   // into the buffer tile t-1 used; everyone is past it now
            const bool mask_next = has_next ? tile_needs_mask(t + 1) : false;

            // ===== sub-tile 1 of tile t: scores in sc[1]
            rescale();
            pv(buf, 0, pf[0]);
#pragma unroll
            for (int x = 0; x < NQT; ++x) softmax(mask_cur, sc[1][x], x, buf, 1, n_valid, pf[1][x]);
            // K.Q of the next tile's first half (past the last tile: recomputed on this tile, result unused)
            qk(has_next ? (t + 1) & (NBUF - 1) : buf, 0, sc[0]);
            mask_cur = mask_next;
        }
        // drain: P.V of the very last sub-tile
        rescale();
        pv((n_tiles - 1) & (NBUF - 1), 1, pf[1]);
    }

    // ---- epilogue: O^T -> LDS -> whole rows to global
    __syncthreads();   // every wave is done with the K/V buffers
    float l_tot[NQT], inv[NQT];
#pragma unroll
    for (int x = 0; x < NQT; ++x) {
        l_tot[x] = sum_across_halves(l_run[x]);
        inv[x] = p.n_splits == 1 ? (l_tot[x] > 0.f ? 1.f / l_tot[x] : 0.f) : 1.f;
    }
    lds_u8 *epi = lds + wave * NQT * 32 * EPI_STRIDE;
#pragma unroll
    for (int x = 0; x < NQT; ++x)
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = o_acc[x][b][i4 * 4 + e] * inv[x];
                *reinterpret_cast<__attribute__((address_space(3))) f32x4 *>(epi + (x * 32 + col) * EPI_STRIDE + (b * 32 + i4 * 8 + hh * 4) * 4) = w;
            }
    // (m, l) of the partial, one lane per query
    if (p.n_splits > 1 && hh == 0) {
#pragma unroll
        for (int x = 0; x < NQT; ++x)
            if (qt[x].valid) {
                const size_t out_row = (size_t)(seq.q_begin + qt[x].qi) * p.Hq + qt[x].head;
                p.part_ml[(size_t)split * p.total_q * p.Hq + out_row] = make_float2(m_run[x], l_tot[x]);
            }
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's LDS writes have landed
    __builtin_amdgcn_wave_barrier();
    // a wave instruction moves 2 rows of 512 bytes (fp32) or 4 rows of 256 bytes (bf16)
#pragma unroll
    for (int x = 0; x < NQT; ++x) {
        // row of the row tile handled by each lane's query index: broadcast through the tile descriptor
        const int rt = rb * kWideRowTilesPerWg + wave * NQT + x;
        if (rt >= row_tiles) continue;
        const int g_head = rt / tiles_q, tq = rt % tiles_q;
        const int head = kvh * p.G + g_head;
        if (p.n_splits > 1) {
#pragma unroll 4
            for (int it = 0; it < 16; ++it) {
                const int q = it * 2 + (lane >> 5);
                const int qi = tq * RW + q;
                const f32x4 w = *reinterpret_cast<const __attribute__((address_space(3))) f32x4 *>(epi + (x * 32 + q) * EPI_STRIDE + (lane & 31) * 16);
                if (qi < seq.n_q) {
                    const size_t out_row = (size_t)(seq.q_begin + qi) * p.Hq + head;
                    float *dst = p.part_o + ((size_t)split * p.total_q * p.Hq + out_row) * D;
                    *reinterpret_cast<f32x4 *>(dst + (lane & 31) * 4) = w;
                }
            }
        } else {
#pragma unroll 4
            for (int it = 0; it < 8; ++it) {
                const int q = it * 4 + (lane >> 4);
                const int qi = tq * RW + q;
                const lds_u8 *src = epi + (x * 32 + q) * EPI_STRIDE + (lane & 15) * 32;
                const f32x4 w0 = *reinterpret_cast<const __attribute__((address_space(3))) f32x4 *>(src);
                const f32x4 w1 = *reinterpret_cast<const __attribute__((address_space(3))) f32x4 *>(src + 16);
                if (qi < seq.n_q) {
                    bf16x8 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) { o[e] = (__bf16)w0[e]; o[4 + e] = (__bf16)w1[e]; }
                    const size_t out_row = (size_t)(seq.q_begin + qi) * p.Hq + head;
                    *reinterpret_cast<bf16x8 *>(p.out + out_row * D + (lane & 15) * 8) = o;
                }
            }
        }
    }
}

template <int NQT, int NW>
int launch_one(pc_ctx *ctx, AttnParams &p, int n_blocks, hipStream_t stream)
{
    static bool attr_set[16] = {false};
    auto kern = attn_bf16_dma_kernel<NQT, NW>;
    if (!attr_set[ctx->device & 15]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                LDS_TOTAL) != hipSuccess)
            return PC_E_HIP;
        attr_set[ctx->device & 15] = true;
    }
    return launch_kernel(ctx, kProfAttn, kern, dim3(n_blocks), dim3(NW * 64), LDS_TOTAL, stream, p);
}

}  // namespace

int launch_attn_bf16_wide(pc_ctx *ctx, attn::AttnParams &p, int n_blocks, int q_tiles_per_wave, hipStream_t stream)
{
    return q_tiles_per_wave == 2 ? launch_one<2, 4>(ctx, p, n_blocks, stream) : launch_one<1, 8>(ctx, p, n_blocks, stream);
}

}  // namespace pc
