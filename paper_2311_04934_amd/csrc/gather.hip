// KV assembly: the "concat" of Sec. 3.4 of the paper as one bandwidth-bound gather.
//
// Every imported module is a contiguous run of rows in the pool (K block, V block);
// the output is the packed concatenation in the order the prompt lists them, plus
// one int32 position ID per row (start_pos + row index).  Bytes are copied verbatim.
//
// Work list: each module's rows are cut into tiles of `rows_per_tile` rows (32 KiB
// of K and 32 KiB of V, twice that for very large launches); the tiles of all segments form one flat list and
// workgroup b takes tile b.  The segment table travels in the kernel arguments, so
// a call needs no host->device copy and no synchronisation.  Each lane moves
// 16 bytes per access and issues all of its loads (K and V) of a pass before the first
// store, which keeps 64 KiB in flight per workgroup.
#include "kv_ops.h"

namespace pc {
namespace {

__global__ __launch_bounds__(kv::kThreads) void gather_kv_kernel(const kv::i32x4 f0, const kv::i32x4 f1, const kv::i32x4 f2,
                                                                  const kv::i32x2 n, const GatherArgs a,
                                                                  uint8_t *__restrict__ out_k, uint8_t *__restrict__ out_v,
                                                                  int32_t *__restrict__ out_pos)
{
    const GatherSeg sg = a.seg[kv::gather_segment(a, n, f0, f1, f2, blockIdx.x)];
    kv::gather_tile_of(a, sg, blockIdx.x, out_k, out_v, out_pos);
}

// The same gather over the modules of several layers: a segment's tiles go to the packed buffers of its layer.
__global__ __launch_bounds__(kv::kThreads) void gather_layers_kernel(const GatherLayersArgs a)
{
    const int si = kv::gather_segment(a.g, blockIdx.x);
    const GatherSeg sg = a.g.seg[si];
    const GatherLayerOut o = a.out[a.seg_layer[si]];
    kv::gather_tile_of(a.g, sg, blockIdx.x, o.k, o.v, o.pos);
}

// Assembly and append in one launch: workgroups [0, total_tiles) gather module rows, the rest append
// one uncached token's row each.  (Every workgroup of such a launch is resident at once; the append
// rows, a chain of dependent loads, run fastest at the end of the grid, when the copy stream drains.)  The two write disjoint rows of the same packed buffers, and a kernel
// launch costs more than the whole append, so a prompt's KV is complete after a single launch.
template <typename T>
__global__ __launch_bounds__(kv::kThreads) void gather_append_kernel(const kv::i32x4 f0, const kv::i32x4 f1, const kv::i32x4 f2,
                                                                      const kv::i32x2 n, const FusedKvArgs a,
                                                                      uint8_t *__restrict__ out_k, uint8_t *__restrict__ out_v,
                                                                      int32_t *__restrict__ out_pos, const T *k_new,
                                                                      const T *v_new, const int32_t *q_pos,
                                                                      int n_kv_heads, int d, const float2 *table,
                                                                      int max_pos, const kv::QRotate<T> qr)
{
    const int b = blockIdx.x;
    if (b < n[1]) {
        const GatherSeg sg = a.g.seg[kv::gather_segment(a.g, n, f0, f1, f2, b)];
        kv::gather_tile_of(a.g, sg, b, out_k, out_v, out_pos);
    } else
        kv::append_row<T>(a.app, a.n_app, b - n[1], k_new, v_new, q_pos, reinterpret_cast<T *>(out_k),
                             reinterpret_cast<T *>(out_v), out_pos, n_kv_heads, d, table, max_pos, qr);
}

}  // namespace

int launch_gather(pc_ctx *ctx, const GatherArgs &args, uint8_t *out_k, uint8_t *out_v, int32_t *out_pos,
                  hipStream_t stream)
{
    if (args.total_tiles <= 0) return PC_OK;
    const kv::GatherHead h = kv::gather_head(args);
    return launch_kernel(ctx, kProfGather, gather_kv_kernel, dim3(args.total_tiles), dim3(kv::kThreads), 0, stream,
                         h.ft[0], h.ft[1], h.ft[2], h.n, args, out_k, out_v, out_pos);
}

int launch_gather_layers(pc_ctx *ctx, const GatherLayersArgs &args, hipStream_t stream)
{
    if (args.g.total_tiles <= 0) return PC_OK;
    return launch_kernel(ctx, kProfGather, gather_layers_kernel, dim3(args.g.total_tiles), dim3(kv::kThreads), 0, stream, args);
}

int launch_gather_append(pc_ctx *ctx, const FusedKvArgs &args, uint8_t *out_k, uint8_t *out_v, int32_t *out_pos,
                         const void *k_new, const void *v_new, const int32_t *q_pos, hipStream_t stream, const void *q_new,
                         void *q_rot, float q_scale)
{
    const int blocks = args.g.total_tiles + args.app_rows;
    if (blocks <= 0) return PC_OK;
    const int n_kv_heads = ctx->cfg.n_kv_heads, head_dim = ctx->cfg.head_dim, max_pos = ctx->cfg.max_pos;
    const float2 *table = ctx->use_alibi ? nullptr : ctx->rope_table;
    const kv::GatherHead h = kv::gather_head(args.g);
    if (ctx->cfg.dtype == PC_F32) {
        kv::QRotate<float> qr;
        qr.q_new = static_cast<const float *>(q_new);
        qr.q_rot = static_cast<float *>(q_rot);
        qr.n_q_heads = ctx->cfg.n_q_heads;
        qr.scale = q_scale;
        return launch_kernel(ctx, kProfGather, gather_append_kernel<float>, dim3(blocks), dim3(kv::kThreads), 0, stream,
                             h.ft[0], h.ft[1], h.ft[2], h.n, args, out_k, out_v, out_pos, static_cast<const float *>(k_new),
                             static_cast<const float *>(v_new), q_pos, n_kv_heads, head_dim, table, max_pos, qr);
    }
    kv::QRotate<uint16_t> qr;
    qr.q_new = static_cast<const uint16_t *>(q_new);
    qr.q_rot = static_cast<uint16_t *>(q_rot);
    qr.n_q_heads = ctx->cfg.n_q_heads;
    qr.scale = q_scale;
    return launch_kernel(ctx, kProfGather, gather_append_kernel<uint16_t>, dim3(blocks), dim3(kv::kThreads), 0, stream,
                         h.ft[0], h.ft[1], h.ft[2], h.n, args, out_k, out_v, out_pos, static_cast<const uint16_t *>(k_new),
                         static_cast<const uint16_t *>(v_new), q_pos, n_kv_heads, head_dim, table, max_pos, qr);
}

}  // namespace pc
