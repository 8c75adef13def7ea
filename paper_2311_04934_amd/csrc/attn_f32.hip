// Uncached-token attention over the assembled KV, fp32 path (Sec. 3.4 of the paper).
//
// Same contract as the bf16 MFMA kernel, everything in fp32 (tolerance 1e-4 against
// an fp64 reference).  One wavefront owns one (query, head) pair: the query is
// rotated at its position ID and parked in LDS; keys are taken 64 at a time, one key
// per lane for the score, then the lanes switch roles and each owns output
// dimensions lane, lane+64, ... for the P.V accumulation.  Online softmax with the
// running maximum and sum kept per wave.
#include <type_traits>

#include "common.h"
#include "kv_seg.h"

namespace pc {
namespace {

constexpr int kWaves = 4;
constexpr int kMaxD = 256;

__device__ __forceinline__ float wave_max_f(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ float wave_sum_f(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

struct F32Params {
    const float *q;
    const int32_t *q_pos;
    const float *k;
    const float *v;
    const int32_t *kv_pos;
    float *out;
    const float2 *rope;
    const float *alibi;  // per-head slopes, or nullptr: rotation
    int q_rotated;       // Q comes rotated and scaled already
    int max_pos, Hq, Hkv, d;
    int q_lo, q_hi;  // query rows covered by this launch
    float scale;
    AttnBatch batch;
};

struct NoTable {
    int unused;
};

// PAGED: K, V and positions are read through the prompt's row ranges (p.k, p.v, p.kv_pos unused).
template <bool PAGED>
__global__ __launch_bounds__(kWaves * 64) void attn_f32_kernel(const F32Params p,
                                                               const std::conditional_t<PAGED, KvSegTable, NoTable> tab)
{
    __shared__ float s_q[kWaves][kMaxD];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long pair = (long)blockIdx.x * kWaves + wave;
    const long n_pairs = (long)(p.q_hi - p.q_lo) * p.Hq;
    const bool in_range = pair < n_pairs;
    const int q_row = p.q_lo + (int)((in_range ? pair : 0) / p.Hq);
    const int h = (int)((in_range ? pair : 0) % p.Hq);
    const int kvh = h / (p.Hq / p.Hkv);
    const int d = p.d, half = d >> 1;

    // which prompt owns this query row
    int si = -1;
    if (in_range)
        for (int s = 0; s < p.batch.n_seqs; ++s)
            if (q_row >= p.batch.seq[s].q_begin && q_row < p.batch.seq[s].q_begin + p.batch.seq[s].n_q) si = s;
    const bool active = si >= 0;
    const AttnSeq seq = p.batch.seq[active ? si : 0];

    // rotate the query at its position ID, fold in 1/sqrt(d)
    const int qpos = active ? p.q_pos[q_row] : 0;
    const float slope = (active && p.alibi) ? p.alibi[h] : 0.f;
    if (active && (p.alibi || p.q_rotated)) {   // linear bias (Sec. 4.2), or Q rotated by the caller: used as it is
        const float *qr = p.q + ((size_t)q_row * p.Hq + h) * d;
        const float sc = p.q_rotated ? 1.f : p.scale;
        for (int i = lane; i < d; i += 64) s_q[wave][i] = qr[i] * sc;
    } else if (active) {
        int tp = qpos < 0 ? 0 : (qpos >= p.max_pos ? p.max_pos - 1 : qpos);
        const float2 *trow = p.rope + (size_t)tp * half;
        const float *qr = p.q + ((size_t)q_row * p.Hq + h) * d;
        for (int i = lane; i < half; i += 64) {
            const float2 cs = trow[i];
            const float lo = qr[i], hi = qr[i + half];
            s_q[wave][i] = (lo * cs.x - hi * cs.y) * p.scale;
            s_q[wave][i + half] = (hi * cs.x + lo * cs.y) * p.scale;
        }
    }
    __syncthreads();
    if (!active) return;
    float *orow = p.out + ((size_t)q_row * p.Hq + h) * d;

    const size_t row_stride = (size_t)p.Hkv * d;
    const float *kb = PAGED ? nullptr : p.k + (size_t)seq.kv_begin * row_stride + (size_t)kvh * d;
    const float *vb = PAGED ? nullptr : p.v + (size_t)seq.kv_begin * row_stride + (size_t)kvh * d;
    const int32_t *pb = PAGED ? nullptr : p.kv_pos + seq.kv_begin;
    KvSegWalker walk;
    if constexpr (PAGED) walk.init(&tab, si);

    float m_run = -INFINITY, l_run = 0.f;
    float acc[kMaxD / 64] = {0.f, 0.f, 0.f, 0.f};

    for (int j0 = 0; j0 < seq.n_kv; j0 += 64) {
        const int j = j0 + lane;
        const float *kr = nullptr, *vr_lane = nullptr;   // this lane's key: its K row and V row (head kvh)
        int kpos = 0;
        if constexpr (PAGED) {
            walk.advance_to((uint32_t)j0);
            const int jc = j < seq.n_kv ? j : seq.n_kv - 1;
            const uint8_t *kp, *vp;
            const int32_t *pp;
            walk.locate((uint32_t)jc, (uint32_t)(j0 + 64 < seq.n_kv ? j0 + 64 : seq.n_kv), (uint32_t)(row_stride * sizeof(float)),
                        (uint32_t)(kvh * d * sizeof(float)), kp, vp, pp);
            kr = reinterpret_cast<const float *>(kp);
            vr_lane = reinterpret_cast<const float *>(vp);
            kpos = *pp;
        } else {
            const int jc = j < seq.n_kv ? j : seq.n_kv - 1;
            kr = kb + (size_t)jc * row_stride;
            vr_lane = vb + (size_t)jc * row_stride;
            kpos = pb[jc];
        }
        const bool vis = j < seq.n_kv && kpos <= qpos;
        float s = -INFINITY;
        if (vis) {
            float dot = 0.f;
            for (int c = 0; c < d; ++c) dot = fmaf(s_q[wave][c], kr[c], dot);
            s = dot - slope * (float)(qpos - kpos);   // slope 0 under rotation
        }
        const float tmax = wave_max_f(s);
        if (tmax == -INFINITY) continue;  // no visible key in these 64 (uniform)
        const float m_new = fmaxf(m_run, tmax);
        const float alpha = expf(m_run - m_new);  // m_run = -inf -> 0
        const float pj = vis ? expf(s - m_new) : 0.f;
        l_run = l_run * alpha + wave_sum_f(pj);
        m_run = m_new;
#pragma unroll
        for (int u = 0; u < kMaxD / 64; ++u) acc[u] *= alpha;
        const int n_here = seq.n_kv - j0 < 64 ? seq.n_kv - j0 : 64;
        for (int kk = 0; kk < n_here; ++kk) {
            const float pk = __shfl(pj, kk, 64);
            if (pk == 0.f) continue;  // uniform: masked or underflowed key contributes nothing
            // V row of key j0 + kk: lane kk holds its address
            const uint64_t va = reinterpret_cast<uint64_t>(vr_lane);
            const float *vr = reinterpret_cast<const float *>(
                ((uint64_t)(uint32_t)__shfl((int)(va >> 32), kk, 64) << 32) | (uint32_t)__shfl((int)(uint32_t)va, kk, 64));
#pragma unroll
            for (int u = 0; u < kMaxD / 64; ++u) {
                const int c = lane + 64 * u;
                if (c < d) acc[u] = fmaf(pk, vr[c], acc[u]);
            }
        }
    }
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
#pragma unroll
    for (int u = 0; u < kMaxD / 64; ++u) {
        const int c = lane + 64 * u;
        if (c < d) orow[c] = acc[u] * inv;
    }
}

}  // namespace

int launch_attn_f32(pc_ctx *ctx, const AttnBatch &batch, const float *q, const int32_t *q_pos, const float *k,
                    const float *v, const int32_t *kv_pos, float *out, hipStream_t stream, const KvSegTable *tab,
                    bool q_rotated)
{
    const int d = ctx->cfg.head_dim;
    if (d > kMaxD || (d & 1)) return PC_E_UNSUPPORTED;
    int q_lo = 1 << 30, q_hi = 0;
    for (int s = 0; s < batch.n_seqs; ++s) {
        if (batch.seq[s].n_q == 0) continue;
        if (batch.seq[s].q_begin < q_lo) q_lo = batch.seq[s].q_begin;
        if (batch.seq[s].q_begin + batch.seq[s].n_q > q_hi) q_hi = batch.seq[s].q_begin + batch.seq[s].n_q;
    }
    if (q_hi <= q_lo) return PC_OK;
    F32Params p;
    p.q = q; p.q_pos = q_pos; p.k = k; p.v = v; p.kv_pos = kv_pos; p.out = out;
    p.rope = ctx->rope_table;
    p.alibi = ctx->use_alibi ? ctx->alibi : nullptr;
    p.q_rotated = q_rotated ? 1 : 0;
    p.max_pos = ctx->cfg.max_pos;
    p.Hq = ctx->cfg.n_q_heads; p.Hkv = ctx->cfg.n_kv_heads; p.d = d;
    p.q_lo = q_lo; p.q_hi = q_hi;
    p.scale = 1.0f / sqrtf((float)d);
    p.batch = batch;
    const long n_pairs = (long)(q_hi - q_lo) * p.Hq;
    const int blocks = (int)((n_pairs + kWaves - 1) / kWaves);
    ctx->last_attn.n_splits = 1;
    ctx->last_attn.n_workgroups = blocks;
    ctx->last_attn.waves_per_wg = kWaves;
    if (tab) return launch_kernel(ctx, kProfAttn, attn_f32_kernel<true>, dim3(blocks), dim3(kWaves * 64), 0, stream, p, *tab);
    return launch_kernel(ctx, kProfAttn, attn_f32_kernel<false>, dim3(blocks), dim3(kWaves * 64), 0, stream, p, NoTable{0});
}

}  // namespace pc
