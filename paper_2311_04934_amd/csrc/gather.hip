// KV assembly: the "concat" of Sec. 3.4 of the paper as one bandwidth-bound gather.
//
// Every imported module is a contiguous run of rows in the pool (K block, V block);
// the output is the packed concatenation in the order the prompt lists them, plus
// one int32 position ID per row (start_pos + row index).  Bytes are copied verbatim.
//
// Work list: each module's rows are cut into tiles of `rows_per_tile` rows (about
// 16 KiB of K and 16 KiB of V); the tiles of all segments form one flat list and
// workgroup b takes tile b.  The segment table travels in the kernel arguments, so
// a call needs no host->device copy and no synchronisation.  Each lane moves
// 16 bytes per access and issues all of its loads (K and V) before the first
// store, which keeps ~32 KiB in flight per workgroup.
#include "common.h"

namespace pc {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kGatherThreads = 256;
constexpr int kUnroll = 4;  // 16-byte accesses per lane per tensor per pass

__global__ __launch_bounds__(kGatherThreads) void gather_kv_kernel(const GatherArgs a, uint8_t *__restrict__ out_k,
                                                                    uint8_t *__restrict__ out_v,
                                                                    int32_t *__restrict__ out_pos)
{
    const int tile = blockIdx.x;
    // segment lookup: last segment whose first_tile <= tile (uniform across the workgroup)
    int lo = 0, hi = a.n_segs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (a.seg[mid].first_tile <= tile) lo = mid;
        else hi = mid - 1;
    }
    const GatherSeg sg = a.seg[lo];
    const int r0 = (tile - sg.first_tile) * a.rows_per_tile;
    int n_rows = sg.n_rows - r0;
    if (n_rows > a.rows_per_tile) n_rows = a.rows_per_tile;
    if (n_rows <= 0) return;

    const size_t src_off = (size_t)r0 * a.row_bytes;
    const size_t dst_off = (size_t)(sg.dst_row + r0) * a.row_bytes;
    const u32x4 *__restrict__ sk = reinterpret_cast<const u32x4 *>(sg.src_k + src_off);
    const u32x4 *__restrict__ sv = reinterpret_cast<const u32x4 *>(sg.src_v + src_off);
    u32x4 *__restrict__ dk = reinterpret_cast<u32x4 *>(out_k + dst_off);
    u32x4 *__restrict__ dv = reinterpret_cast<u32x4 *>(out_v + dst_off);
    const int n_vec = (int)(((size_t)n_rows * a.row_bytes) >> 4);

    for (int base = 0; base < n_vec; base += kGatherThreads * kUnroll) {
        u32x4 rk[kUnroll], rv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int i = base + u * kGatherThreads + threadIdx.x;
            if (i < n_vec) {
                rk[u] = __builtin_nontemporal_load(sk + i);
                rv[u] = __builtin_nontemporal_load(sv + i);
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int i = base + u * kGatherThreads + threadIdx.x;
            if (i < n_vec) {
                dk[i] = rk[u];
                dv[i] = rv[u];
            }
        }
    }
    for (int r = threadIdx.x; r < n_rows; r += kGatherThreads)
        out_pos[sg.dst_row + r0 + r] = sg.start_pos + r0 + r;
}

}  // namespace

int launch_gather(pc_ctx *ctx, const GatherArgs &args, uint8_t *out_k, uint8_t *out_v, int32_t *out_pos,
                  hipStream_t stream)
{
    if (args.total_tiles <= 0) return PC_OK;
    return launch_kernel(ctx, kProfGather, gather_kv_kernel, dim3(args.total_tiles), dim3(kGatherThreads), 0, stream,
                         args, out_k, out_v, out_pos);
}

}  // namespace pc
