// Uncached-token prefill attention over the assembled KV, bf16 MFMA path (gfx950).
//
// Computes, for every uncached query q and query head h (Sec. 3.4 of the paper:
// the uncached tokens run through attention with the concatenated module states
// as their KV cache):
//     out[q][h] = sum_j softmax_j( rope(Q[q][h], q_pos[q]) . K[j][kv(h)] / sqrt(d) ) V[j][kv(h)]
// over the rows j whose schema position ID is <= q_pos[q].
//
// Decomposition
//   work unit  = (prompt, kv head, KV split, row block)
//   row tile   = 32 queries of one query head; one wavefront owns one row tile for
//                the whole kernel.  The query heads that share a kv head (GQA) are
//                stacked: a workgroup's NW waves take NW row tiles of the same kv
//                head, so each K/V tile is fetched once per workgroup and used by
//                all of them.
//   KV tile    = 64 keys, staged through LDS (double buffered): K row-major with a
//                16-byte pad per row, V transposed on the way in so that the PV
//                MFMA reads 8 consecutive keys per lane with one 16-byte LDS load.
//   MFMA       v_mfma_f32_32x32x16_bf16.  Scores are produced TRANSPOSED
//                (S^T = K . Q^T: rows = keys, columns = queries) so that every lane
//                owns one query column: the softmax row reductions are 16 in-lane
//                values plus one exchange with lane^32, and P^T in the accumulator
//                layout is directly the B operand of  O^T += V^T . P^T.
//   softmax    online, base 2 (log2(e)/sqrt(d) is folded into Q), fp32 statistics;
//                P is rounded to bf16 for the PV product.
//   mask       per key tile the min/max position ID decides "all visible",
//                "none visible" (tile skipped) or "mixed" (per-element compare).
//   split-KV   when one pass would not fill the GPU, the key range is cut into
//                n_splits pieces; partial (m, l) in fp32 and O in bf16 go to scratch and
//                a merge kernel combines them by log-sum-exp.
//   XCD        workgroups are handed out round-robin over the 8 XCDs, so the group
//                index is laid out such that all row blocks of one (kv head, split)
//                land on the same XCD and share its L2.

#include <type_traits>

#include "attn_bf16.h"

namespace pc {
namespace {

using namespace attn;

template <int D>
struct Lds {
    static constexpr int K_STRIDE = D * 2 + 16;        // bytes per K row (padded)
    static constexpr int V_STRIDE = KT * 2 + 16;       // bytes per V^T row (padded)
    static constexpr int K_BYTES = KT * K_STRIDE;
    static constexpr int V_BYTES = D * V_STRIDE;
    static constexpr int POS_BYTES = KT * 4;
    static constexpr int META_BYTES = 16;
    static constexpr int BUF_BYTES = K_BYTES + V_BYTES + POS_BYTES + META_BYTES;
    static constexpr int TOTAL = 2 * BUF_BYTES;
};

// 4x4 transpose of 16-bit values held as four (lo,hi) dword pairs: in[e] = 4 dims of key e,
// out[i] = 4 keys of dim i.
__device__ __forceinline__ void transpose4x4_b16(const u32x2 in[4], u32x2 out[4])
{
    out[0].x = (in[0].x & 0xffffu) | (in[1].x << 16);
    out[0].y = (in[2].x & 0xffffu) | (in[3].x << 16);
    out[1].x = (in[0].x >> 16) | (in[1].x & 0xffff0000u);
    out[1].y = (in[2].x >> 16) | (in[3].x & 0xffff0000u);
    out[2].x = (in[0].y & 0xffffu) | (in[1].y << 16);
    out[2].y = (in[2].y & 0xffffu) | (in[3].y << 16);
    out[3].x = (in[0].y >> 16) | (in[1].y & 0xffff0000u);
    out[3].y = (in[2].y >> 16) | (in[3].y & 0xffff0000u);
}

// Registers that carry one K/V tile from global memory to LDS.
template <int D, int NW>
struct TileRegs {
    static constexpr int NT = NW * 64;
    static constexpr int K_PER_T = (KT * D / 8 + NT - 1) / NT;
    static constexpr int V_PER_T = (16 * (D / 4) + NT - 1) / NT;
    u32x4 k[K_PER_T];
    u32x2 v[V_PER_T][4];
    int pos;
};

struct NoTable {
    int unused;
};

// PAGED: K, V and positions are read through the prompt's row ranges (p.k, p.v, p.kv_pos unused).
template <int D, int NW, bool PAGED>
__global__ __launch_bounds__(NW * 64) void attn_bf16_kernel(const AttnParams p,
                                                            const std::conditional_t<PAGED, KvSegTable, NoTable> tab)
{
    constexpr int NT = NW * 64;
    constexpr int KB = D / 16;              // MFMA k-blocks over the head dim (QK^T)
    constexpr int DB = D / 32;              // 32-row blocks of O^T
    constexpr int K_CHUNKS = KT * D / 8;    // 16-byte chunks in a K tile
    constexpr int V_BLOCKS = 16 * (D / 4);  // 4-key x 4-dim blocks in a V tile
    using L = Lds<D>;
    using Regs = TileRegs<D, NW>;

    extern __shared__ __align__(16) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;   // query column inside the row tile
    const int hh = lane >> 5;    // which half of the wave

    // ---- which work unit (XCD-aware: consecutive block ids go to consecutive XCDs)
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int g = (slot / p.rb_max) * 8 + xcd;
    const int rb = slot % p.rb_max;
    if (g >= p.n_groups) return;
    // kv head fastest: the KV splits of a (prompt, kv head) share an XCD, hence its L2 copy of their query rows
    const int kvh = g % p.Hkv;
    const int split = (g / p.Hkv) % p.n_splits;
    const int seq_i = g / (p.Hkv * p.n_splits);
    AttnSeq seq = p.seq0;
    if (p.n_seqs > 1) seq = p.batch.seq[seq_i];

    const int tiles_q = (seq.n_q + RW - 1) / RW;
    const int row_tiles = p.G * tiles_q;
    if (rb * NW >= row_tiles) return;   // whole workgroup has nothing to do

    // this split's key range: equal shares rounded up to whole 64-key tiles (only a prompt's last split ends ragged)
    const int share = (((seq.n_kv + p.n_splits - 1) / p.n_splits) + KT - 1) & ~(KT - 1);
    const int k_begin = split * share < seq.n_kv ? split * share : seq.n_kv;
    const int k_end = k_begin + share < seq.n_kv ? k_begin + share : seq.n_kv;
    const int n_tiles = (k_end - k_begin + KT - 1) / KT;

    // ---- this wave's row tile
    const int rt = rb * NW + wave;
    const bool wave_active = rt < row_tiles;
    const int g_head = wave_active ? rt / tiles_q : 0;
    const int qt = wave_active ? rt % tiles_q : 0;
    const int head = kvh * p.G + g_head;
    const int qi = qt * RW + col;                       // query index inside the prompt
    const bool q_valid = wave_active && qi < seq.n_q;
    const int q_row = seq.q_begin + (q_valid ? qi : 0);  // clamped for loads
    const int my_qpos = q_valid ? p.q_pos[q_row] : kPosInf;

    // ---- prologue: load Q, rotate at the query's position ID, scale, round to bf16
    bf16x8 qf[KB];
    {
        const uint16_t *qrow = p.q + ((size_t)q_row * p.Hq + head) * D;
        int tpos = my_qpos;
        tpos = tpos < 0 ? 0 : (tpos >= p.max_pos ? p.max_pos - 1 : tpos);
        const float2 *trow = p.rope + (size_t)tpos * (D / 2);
#pragma unroll
        for (int kb = 0; kb < KB / 2; ++kb) {
            const int d0 = kb * 16 + hh * 8;  // < D/2
            u32x4 lo = *reinterpret_cast<const u32x4 *>(qrow + d0);
            u32x4 hi = *reinterpret_cast<const u32x4 *>(qrow + d0 + D / 2);
            bf16x8 olo, ohi;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint32_t wl = lo[e >> 1], wh = hi[e >> 1];
                float xl = bf16_bits_to_f32((e & 1) ? (wl >> 16) : (wl & 0xffffu));
                float xh = bf16_bits_to_f32((e & 1) ? (wh >> 16) : (wh & 0xffffu));
                float2 cs = (p.alibi || p.q_rotated) ? make_float2(1.f, 0.f) : trow[d0 + e];   // linear bias or rotated by the caller: Q as it is
                const float qs = p.q_rotated ? 1.f : p.q_scale;
                olo[e] = (__bf16)((xl * cs.x - xh * cs.y) * qs);
                ohi[e] = (__bf16)((xh * cs.x + xl * cs.y) * qs);
            }
            qf[kb] = olo;
            qf[kb + KB / 2] = ohi;
        }
    }
    const float slope2 = p.alibi ? p.alibi[head] * 1.4426950408889634f : 0.f;
    // position range of this wave's real queries (decides masking per key tile)
    const int wave_min_qpos = wave_min_i32(q_valid ? my_qpos : kPosInf);
    const int wave_max_qpos = wave_max_i32(q_valid ? my_qpos : -1);

    // ---- accumulators
    f32x16 o_acc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[b][i] = 0.f;
    float m_run = -INFINITY;  // running max (log2 domain), identical in both halves of the wave
    float l_run = 0.f;        // this lane's share of the running sum (halves added at the end)

    const size_t kv_row_stride = (size_t)p.Hkv * D;  // elements
    const uint16_t *k_base = PAGED ? nullptr : p.k + (size_t)seq.kv_begin * kv_row_stride + (size_t)kvh * D;
    const uint16_t *v_base = PAGED ? nullptr : p.v + (size_t)seq.kv_begin * kv_row_stride + (size_t)kvh * D;
    const int32_t *pos_base = PAGED ? nullptr : p.kv_pos + seq.kv_begin;
    KvSegWalker walk;
    if constexpr (PAGED) walk.init(&tab, seq_i);
    // PAGED: first byte of row `rc` of this kv head in K and in V, and the row's position ID
    auto row_ptrs = [&](int rc, int row_hi, const uint16_t *&kp, const uint16_t *&vp, const int32_t *&pp) {
        if constexpr (PAGED) {
            const uint8_t *k8, *v8;
            walk.locate((uint32_t)rc, (uint32_t)row_hi, (uint32_t)(kv_row_stride * 2), (uint32_t)(kvh * D * 2), k8, v8, pp);
            kp = reinterpret_cast<const uint16_t *>(k8);
            vp = reinterpret_cast<const uint16_t *>(v8);
        } else {
            kp = k_base + (size_t)rc * kv_row_stride;
            vp = v_base + (size_t)rc * kv_row_stride;
            pp = pos_base + rc;
        }
    };

    // global -> registers.  Branch-free: rows at or past k_end are read from the last valid row
    // and then zeroed (position +inf), so all loads of a tile are in flight together.
    auto load_tile = [&](int t, Regs &r) {
        const int row0 = k_begin + t * KT;
        const int last = k_end - 1;
        const int row_hi = row0 + KT < k_end ? row0 + KT : k_end;
        if constexpr (PAGED) walk.advance_to((uint32_t)(row0 < last ? row0 : last));
        const uint16_t *kp, *vp;
        const int32_t *pp;
#pragma unroll
        for (int it = 0; it < Regs::K_PER_T; ++it) {
            const int c = tid + it * NT;
            if (K_CHUNKS % NT == 0 || c < K_CHUNKS) {
                const int row = row0 + c / (D / 8), ch = c % (D / 8);
                const int rc = row < last ? row : last;
                row_ptrs(rc, row_hi, kp, vp, pp);
                u32x4 val = *reinterpret_cast<const u32x4 *>(kp + ch * 8);
                if (row > last) val = u32x4{0u, 0u, 0u, 0u};
                r.k[it] = val;
            }
        }
#pragma unroll
        for (int it = 0; it < Regs::V_PER_T; ++it) {
            const int c = tid + it * NT;
            if (V_BLOCKS % NT == 0 || c < V_BLOCKS) {
                const int dc = c % (D / 4), kg = c / (D / 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = row0 + kg * 4 + e;
                    const int rc = row < last ? row : last;
                    row_ptrs(rc, row_hi, kp, vp, pp);
                    u32x2 val = *reinterpret_cast<const u32x2 *>(vp + dc * 4);
                    if (row > last) val = u32x2{0u, 0u};
                    r.v[it][e] = val;
                }
            }
        }
        {   // every wave reads the tile's 64 position IDs (one per lane); wave 0's copy is the one stored
            const int row = row0 + lane;
            const int rc = row < last ? row : last;
            row_ptrs(rc, row_hi, kp, vp, pp);
            const int pv = *pp;
            r.pos = row > last ? kPosInf : pv;
        }
    };

    // registers -> LDS (K as is, V transposed, positions and their range)
    auto store_tile = [&](int buf, const Regs &r) {
        uint8_t *sK = smem + buf * L::BUF_BYTES;
        uint8_t *sV = sK + L::K_BYTES;
        int32_t *sPos = reinterpret_cast<int32_t *>(sV + L::V_BYTES);
        int32_t *sMeta = sPos + KT;
#pragma unroll
        for (int it = 0; it < Regs::K_PER_T; ++it) {
            const int c = tid + it * NT;
            const int rr = c / (D / 8), ch = c % (D / 8);
            if (K_CHUNKS % NT == 0 || c < K_CHUNKS) *reinterpret_cast<u32x4 *>(sK + rr * L::K_STRIDE + ch * 16) = r.k[it];
        }
#pragma unroll
        for (int it = 0; it < Regs::V_PER_T; ++it) {
            const int c = tid + it * NT;
            const int dc = c % (D / 4), kg = c / (D / 4);
            if (V_BLOCKS % NT == 0 || c < V_BLOCKS) {
                u32x2 tr[4];
                transpose4x4_b16(r.v[it], tr);
                // keys 4*kg .. 4*kg+3 of the tile; inside each block of 16 keys the four
                // 4-key groups are stored in the order 0,2,1,3 so that the 8 keys a lane
                // needs for one PV MFMA are contiguous
                const int blk = kg >> 2, g4 = kg & 3;
                const int sg = ((g4 & 1) << 1) | (g4 >> 1);
                const int slot0 = blk * 16 + sg * 4;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    *reinterpret_cast<u32x2 *>(sV + (dc * 4 + i) * L::V_STRIDE + slot0 * 2) = tr[i];
            }
        }
        if (tid < KT) {
            sPos[tid] = r.pos;
            // wave 0 holds all 64 position IDs of the tile: publish their range
            const int real_min = wave_min_i32(r.pos);  // padding is +inf
            const int real_max = wave_max_i32(r.pos);  // +inf if any padding
            if (tid == 0) { sMeta[0] = real_min; sMeta[1] = real_max; }
        }
    };

    // S^T (32 keys x 32 queries) = K_sub . Q^T for one 32-key half of the tile
    auto qk = [&](const uint8_t *sK, int sub) -> f32x16 {
        f32x16 s;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
        const uint8_t *krow = sK + (sub * 32 + col) * L::K_STRIDE + hh * 16;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            u32x4 raw = *reinterpret_cast<const u32x4 *>(krow + kb * 32);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), qf[kb], s, 0, 0, 0);
        }
        return s;
    };

    // mask (if needed) + online softmax of one score tile; rescales O when the running max moved
    auto softmax = [&](f32x16 &s, const int32_t *sPos, int sub, bool need_mask, bf16x8 pf[2]) {
        if (p.alibi) {
            // linear bias on position IDs (Sec. 4.2): + slope * (pos_k - ref) in the log2 domain; the part that
            // depends on the query only is constant per softmax row and is left out
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const u32x4 kp = *reinterpret_cast<const u32x4 *>(sPos + sub * 32 + 8 * i4 + 4 * hh);
#pragma unroll
                for (int e = 0; e < 4; ++e) s[i4 * 4 + e] += slope2 * (float)((int)kp[e] - wave_min_qpos);
            }
        }
        if (need_mask) {
            // accumulator register i holds key 8*(i/4) + 4*hh + i%4 of the sub-tile
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const u32x4 kp = *reinterpret_cast<const u32x4 *>(sPos + sub * 32 + 8 * i4 + 4 * hh);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((int)kp[e] > my_qpos) s[i4 * 4 + e] = -INFINITY;
            }
        }
        float mx = s[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i]);
        mx = max_across_halves(mx);
        const float m_new = mx > m_run + kMaxSlack ? mx : m_run;
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float pv = __builtin_amdgcn_exp2f(s[i] - m_use);
            psum += pv;
            pf[i >> 3][i & 7] = (__bf16)pv;
        }
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) o_acc[b][i] *= alpha;
        }
    };

    // O^T (D x 32 queries) += V^T_sub . P^T
    auto pv_mma = [&](const uint8_t *sV, int sub, const bf16x8 pf[2]) {
        const uint8_t *vrow = sV + col * L::V_STRIDE + (sub * 2) * 32 + hh * 16;
#pragma unroll
        for (int b = 0; b < DB; ++b) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                u32x4 raw = *reinterpret_cast<const u32x4 *>(vrow + b * 32 * L::V_STRIDE + j * 32);
                o_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), pf[j], o_acc[b], 0, 0, 0);
            }
        }
    };

    // One 64-key tile.  Both score tiles are issued before the first softmax so that the matrix
    // pipe works on the second while the vector ALU runs the first one's softmax.
    auto compute_tile = [&](int buf, int t) {
        const uint8_t *sK = smem + buf * L::BUF_BYTES;
        const uint8_t *sV = sK + L::K_BYTES;
        const int32_t *sPos = reinterpret_cast<const int32_t *>(sV + L::V_BYTES);
        const int32_t *sMeta = sPos + KT;
        const int tile_min = __builtin_amdgcn_readfirstlane(sMeta[0]);
        const int tile_max = __builtin_amdgcn_readfirstlane(sMeta[1]);
        if (tile_min > wave_max_qpos) return;             // nothing in this tile is visible to this wave
        const bool need_mask = tile_max > wave_min_qpos;  // some (query, key) pair is hidden
        const bool second = k_begin + t * KT + 32 < k_end;  // the tile's second half holds real keys
        bf16x8 pf[2];
        f32x16 s0 = qk(sK, 0);
        if (second) {
            f32x16 s1 = qk(sK, 1);
            softmax(s0, sPos, 0, need_mask, pf);
            pv_mma(sV, 0, pf);
            softmax(s1, sPos, 1, need_mask, pf);
            pv_mma(sV, 1, pf);
        } else {
            softmax(s0, sPos, 0, need_mask, pf);
            pv_mma(sV, 0, pf);
        }
    };

    // ---- main loop: LDS double buffer; the global loads of tile t+1 are in flight while tile t is computed
    if (n_tiles > 0) {
        Regs ra;
        load_tile(0, ra);
        store_tile(0, ra);
        __syncthreads();
        for (int t = 0; t < n_tiles; ++t) {
            const bool more = t + 1 < n_tiles;
            if (more) load_tile(t + 1, ra);
            if (wave_active) compute_tile(t & 1, t);
            if (more) store_tile((t + 1) & 1, ra);
            __syncthreads();
        }
    }

    // ---- epilogue
    if (!q_valid) return;
    const float l_tot = sum_across_halves(l_run);
    const size_t out_row = (size_t)(seq.q_begin + qi) * p.Hq + head;
    if (p.n_splits == 1) {
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        uint16_t *orow = p.out + out_row * D;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o_acc[b][i4 * 4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(orow + b * 32 + i4 * 8 + hh * 4) = w;
            }
    } else {
        const size_t prow = (size_t)split * p.total_q * p.Hq + out_row;
        uint16_t *orow = p.part_o + prow * D;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (__bf16)o_acc[b][i4 * 4 + e];
                *reinterpret_cast<bf16x4 *>(orow + b * 32 + i4 * 8 + hh * 4) = w;
            }
        if (hh == 0) p.part_ml[prow] = make_float2(m_run, l_tot);
    }
}

// Merge the split-KV partials: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.  The partial O_s are
// stored in bf16 (they are rounded to bf16 at the output anyway, and the merge is a convex
// combination); m_s and l_s are fp32.  One thread owns 8 elements of a row.  HEAD_MAJOR: the partials of a split
// are [Hq][total_q] rows (the DMA-staged kernel's), else [total_q][Hq] like the output.
template <int D, bool HEAD_MAJOR>
__global__ __launch_bounds__(256) void attn_combine_kernel(const uint16_t *part_o, const float2 *part_ml, uint16_t *out,
                                                           int n_splits, long n_rows /* total_q * Hq */,
                                                           long row_lo, long row_hi /* rows this launch owns */, int Hq)
{
    constexpr int CH = D / 8;  // 8-element chunks per row
    constexpr int U = 8;       // splits fetched together: all their loads are in flight at once
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (row_hi - row_lo) * CH) return;
    const long row = row_lo + idx / CH;
    const int ch = (int)(idx % CH);
    const long prow = HEAD_MAJOR ? (row % Hq) * (n_rows / Hq) + row / Hq : row;   // row of one split's partials
    float M = -INFINITY, Lsum = 0.f;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int s0 = 0; s0 < n_splits; s0 += U) {
        float2 ml[U];
        u32x4 o[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = s0 + u < n_splits ? s0 + u : n_splits - 1;   // clamped: a repeated split gets weight 0 below
            ml[u] = part_ml[(size_t)s * n_rows + prow];
            o[u] = *reinterpret_cast<const u32x4 *>(part_o + ((size_t)s * n_rows + prow) * D + ch * 8);
        }
        float Mg = M;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (s0 + u < n_splits) Mg = fmaxf(Mg, ml[u].x);
        if (Mg == -INFINITY) continue;            // nothing visible so far
        const float r = __builtin_amdgcn_exp2f(M - Mg);   // M = -inf gives 0, and acc and Lsum are 0 then
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= r;
        Lsum *= r;
        M = Mg;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // a split that saw no visible key has m = -inf and an O that may be unset: it is skipped
            const bool use = s0 + u < n_splits && ml[u].x != -INFINITY;
            const float w = use ? __builtin_amdgcn_exp2f(ml[u].x - M) : 0.f;
            Lsum += use ? w * ml[u].y : 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t word = o[u][e >> 1];
                const float x = bf16_bits_to_f32((e & 1) ? (word >> 16) : (word & 0xffffu));
                acc[e] += use ? x * w : 0.f;
            }
        }
    }
    const float inv = Lsum > 0.f ? 1.f / Lsum : 0.f;
    bf16x8 w8;
#pragma unroll
    for (int e = 0; e < 8; ++e) w8[e] = (__bf16)(acc[e] * inv);
    *reinterpret_cast<bf16x8 *>(out + (size_t)row * D + ch * 8) = w8;
}

template <int D, int NW, bool PAGED = false, typename Tab = NoTable>
int launch_variant(pc_ctx *ctx, AttnParams &p, int n_blocks, hipStream_t stream, const Tab &tab = NoTable{0})
{
    static bool attr_set[16] = {false};
    auto kern = attn_bf16_kernel<D, NW, PAGED>;
    const int smem = Lds<D>::TOTAL;
    if (!attr_set[ctx->device & 15]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return PC_E_HIP;
        attr_set[ctx->device & 15] = true;
    }
    return launch_kernel(ctx, kProfAttn, kern, dim3(n_blocks), dim3(NW * 64), smem, stream, p, tab);
}

}  // namespace

int launch_attn_bf16(pc_ctx *ctx, const AttnBatch &batch, const void *q, const int32_t *q_pos, const void *k,
                     const void *v, const int32_t *kv_pos, void *out, hipStream_t stream, const KvSegTable *tab, bool q_rotated,
                     const ScratchRef *scratch)
{
    const ScratchRef own{reinterpret_cast<uint8_t *>(ctx->scratch), ctx->scratch_bytes, false};
    const ScratchRef &sc = scratch ? *scratch : own;
    const int D = ctx->cfg.head_dim, Hq = ctx->cfg.n_q_heads, Hkv = ctx->cfg.n_kv_heads, G = Hq / Hkv;
    if (D != 64 && D != 128) return PC_E_UNSUPPORTED;

    int total_q = 0, q_lo = 1 << 30, max_row_tiles = 0, min_kv = 1 << 30;
    for (int s = 0; s < batch.n_seqs; ++s) {
        const AttnSeq &sq = batch.seq[s];
        total_q = sq.q_begin + sq.n_q > total_q ? sq.q_begin + sq.n_q : total_q;
        q_lo = sq.q_begin < q_lo ? sq.q_begin : q_lo;
        const int rt = G * ((sq.n_q + RW - 1) / RW);
        if (rt > max_row_tiles) max_row_tiles = rt;
        if (sq.n_q > 0 && sq.n_kv < min_kv) min_kv = sq.n_kv;
    }
    if (total_q == 0 || max_row_tiles == 0) return PC_OK;

    // DMA-staged kernel: every head_dim-128 call whose packed buffer fits 32-bit row offsets (or is read in place)
    long max_kv = 0;
    for (int s = 0; s < batch.n_seqs; ++s) max_kv = batch.seq[s].n_kv > max_kv ? batch.seq[s].n_kv : max_kv;
    const bool fits_u32 = max_kv * (long)Hkv * D * 2 < (1L << 32);   // the wide kernel uses 32-bit row offsets
    // a range table is read by the DMA-staged kernel only (32-bit offsets there are per range, checked by the caller)
    const bool wide = D == 128 && (tab || (max_row_tiles >= kWideMinRowTiles && fits_u32 && ctx->attn_kernel == PC_ATTN_AUTO));
    const int NW = wide ? 4 : (max_row_tiles <= 4 ? 4 : 8);
    const int tiles_per_wg = wide ? kWideRowTilesPerWg : NW;
    const int rb_max = (max_row_tiles + tiles_per_wg - 1) / tiles_per_wg;
    const long base_wgs = (long)batch.n_seqs * Hkv * rb_max;
    const long target = wide ? (long)ctx->n_cu : (long)ctx->n_cu * (8 / NW);

    // KV splits: enough workgroups to fill the GPU, at least 128 keys per split,
    // and the partials must fit the scratch.
    int n_splits = (int)((target + base_wgs - 1) / base_wgs);
    const int max_by_keys = min_kv / 128 > 1 ? min_kv / 128 : 1;
    if (n_splits > max_by_keys) n_splits = max_by_keys;
    if (n_splits > 32) n_splits = 32;
    if (n_splits < 1) n_splits = 1;
    // A split's share is a whole number of 64-key tiles (the kernels round it up), so with T tiles in the longest
    // prompt only ceil(T / ceil(T / n_splits)) splits get any keys: launch exactly those.  The others would run a
    // prologue and write partials that the merge then reads for nothing.
    if (n_splits > 1) {
        const int longest = (int)((max_kv + KT - 1) / KT);
        const int tiles_per_split = (longest + n_splits - 1) / n_splits;
        n_splits = (longest + tiles_per_split - 1) / tiles_per_split;
    }
    // partial O of every split, padded to 256 bytes, then every split's (m, l)
    auto ml_offset = [&](int ns) { return ((size_t)ns * total_q * Hq * D * sizeof(uint16_t) + 255) & ~(size_t)255; };
    auto scratch_need = [&](int ns) { return ml_offset(ns) + (size_t)ns * total_q * Hq * sizeof(float2); };
    if (n_splits > 1 && scratch_need(n_splits) > sc.bytes) {
        if (sc.strict) return PC_E_CAPACITY;
        while (n_splits > 1 && scratch_need(n_splits) > sc.bytes) --n_splits;
    }

    AttnParams p;
    p.q = static_cast<const uint16_t *>(q);
    p.q_pos = q_pos;
    p.k = static_cast<const uint16_t *>(k);
    p.v = static_cast<const uint16_t *>(v);
    p.kv_pos = kv_pos;
    p.out = static_cast<uint16_t *>(out);
    p.part_o = reinterpret_cast<uint16_t *>(sc.ptr);
    p.part_ml = reinterpret_cast<float2 *>(sc.ptr + ml_offset(n_splits));
    p.rope = ctx->rope_table;
    p.rope_t = ctx->rope_table_t;
    p.alibi = ctx->use_alibi ? ctx->alibi : nullptr;
    p.q_rotated = q_rotated ? 1 : 0;
    p.max_pos = ctx->cfg.max_pos;
    p.Hq = Hq;
    p.Hkv = Hkv;
    p.G = G;
    p.n_splits = n_splits;
    p.rb_max = rb_max;
    p.n_groups = batch.n_seqs * n_splits * Hkv;
    p.total_q = total_q;
    p.q_scale = 1.4426950408889634f / sqrtf((float)D);
    p.batch = batch;
    p.n_seqs = batch.n_seqs;
    p.seq0 = p.batch.seq[0];

    const int n_blocks = 8 * ((p.n_groups + 7) / 8) * rb_max;
    int rc;
    int waves_used = NW;
    if (wide) {
        rc = launch_attn_bf16_wide(ctx, p, n_blocks, stream, tab);
        waves_used = 8;
    } else if (D == 128) {
        rc = NW == 8 ? launch_variant<128, 8>(ctx, p, n_blocks, stream) : launch_variant<128, 4>(ctx, p, n_blocks, stream);
    } else if (tab) {   // head_dim 64 read in place
        rc = NW == 8 ? launch_variant<64, 8, true>(ctx, p, n_blocks, stream, *tab) : launch_variant<64, 4, true>(ctx, p, n_blocks, stream, *tab);
    } else {
        rc = NW == 8 ? launch_variant<64, 8>(ctx, p, n_blocks, stream) : launch_variant<64, 4>(ctx, p, n_blocks, stream);
    }
    if (rc != PC_OK) return rc;

    if (n_splits > 1) {
        // the prompts of one launch own the contiguous query rows [q_lo, total_q)
        const long n_rows = (long)total_q * Hq;
        const long row_lo = (long)q_lo * Hq;
        const long n_thr = (n_rows - row_lo) * (D / 8);
        const int blocks = (int)((n_thr + 255) / 256);
        const uint16_t *po = p.part_o;
        const float2 *pml = p.part_ml;
        if (wide)
            rc = launch_kernel(ctx, kProfCombine, attn_combine_kernel<128, true>, dim3(blocks), dim3(256), 0, stream, po, pml,
                               p.out, n_splits, n_rows, row_lo, n_rows, Hq);
        else if (D == 128)
            rc = launch_kernel(ctx, kProfCombine, attn_combine_kernel<128, false>, dim3(blocks), dim3(256), 0, stream, po, pml,
                               p.out, n_splits, n_rows, row_lo, n_rows, Hq);
        else
            rc = launch_kernel(ctx, kProfCombine, attn_combine_kernel<64, false>, dim3(blocks), dim3(256), 0, stream, po, pml,
                               p.out, n_splits, n_rows, row_lo, n_rows, Hq);
    }
    ctx->last_attn.n_splits = n_splits;
    ctx->last_attn.n_workgroups = n_blocks;
    ctx->last_attn.waves_per_wg = waves_used;
    return rc;
}

}  // namespace pc
