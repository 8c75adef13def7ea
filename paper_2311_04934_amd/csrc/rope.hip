// RoPE at arbitrary position IDs, and the append of the uncached tokens' own K/V.
//
// Prompt modules are encoded at the position IDs their schema fixes, which do not
// start at zero and are not contiguous across a prompt (Sec. 3.3 of the paper);
// the rotation is therefore looked up by position ID in a table (Sec. 4.2).  The
// table holds (cos, sin) of pos * base^(-2i/d), computed in fp64 on the host and
// rounded once to fp32, so the angle carries no fp32 range-reduction error even
// at positions in the tens of thousands.  Pairing is half-split: element i rotates
// with element i + d/2.
#include "kv_ops.h"

namespace pc {
namespace {

using kv::clamp_pos;
using kv::Elem;

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

// One workgroup per appended row (see kv::append_row).
template <typename T>
__global__ __launch_bounds__(kv::kThreads) void append_kernel(const AppendArgs a, const T *k_new, const T *v_new,
                                                              const int32_t *q_pos, T *asm_k, T *asm_v,
                                                              int32_t *asm_pos, int n_kv_heads, int d,
                                                              const float2 *table, int max_pos, const kv::QRotate<T> qr)
{
    kv::append_row<T>(a.seg, a.n_segs, blockIdx.x, k_new, v_new, q_pos, asm_k, asm_v, asm_pos, n_kv_heads, d, table,
                      max_pos, qr);
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
                  void *asm_k, void *asm_v, int32_t *asm_pos, hipStream_t stream, const void *q_new, void *q_rot,
                  float q_scale)
{
    if (args.total_rows <= 0) return PC_OK;
    const int n_kv_heads = ctx->cfg.n_kv_heads, head_dim = ctx->cfg.head_dim, max_pos = ctx->cfg.max_pos;
    const float2 *table = ctx->use_alibi ? nullptr : ctx->rope_table;   // linear-bias models store keys unrotated
    if (ctx->cfg.dtype == PC_F32) {
        kv::QRotate<float> qr;
        qr.q_new = static_cast<const float *>(q_new);
        qr.q_rot = static_cast<float *>(q_rot);
        qr.n_q_heads = ctx->cfg.n_q_heads;
        qr.scale = q_scale;
        return launch_kernel(ctx, kProfAppend, append_kernel<float>, dim3(args.total_rows), dim3(kv::kThreads), 0, stream, args,
                             static_cast<const float *>(k_new), static_cast<const float *>(v_new), q_pos,
                             static_cast<float *>(asm_k), static_cast<float *>(asm_v), asm_pos, n_kv_heads, head_dim,
                             table, max_pos, qr);
    }
    kv::QRotate<uint16_t> qr;
    qr.q_new = static_cast<const uint16_t *>(q_new);
    qr.q_rot = static_cast<uint16_t *>(q_rot);
    qr.n_q_heads = ctx->cfg.n_q_heads;
    qr.scale = q_scale;
    return launch_kernel(ctx, kProfAppend, append_kernel<uint16_t>, dim3(args.total_rows), dim3(kv::kThreads), 0, stream, args,
                         static_cast<const uint16_t *>(k_new), static_cast<const uint16_t *>(v_new), q_pos,
                         static_cast<uint16_t *>(asm_k), static_cast<uint16_t *>(asm_v), asm_pos, n_kv_heads, head_dim,
                         table, max_pos, qr);
}

}  // namespace pc
