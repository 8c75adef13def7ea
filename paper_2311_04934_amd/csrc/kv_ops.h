// Device bodies of the KV assembly: the gather of one tile of module rows and the append of one
// uncached token's row.  Shared by the stand-alone kernels and the fused assemble+append kernel.
#pragma once
#include "common.h"

namespace pc {
namespace kv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kUnroll = 4;  // 16-byte accesses per lane per tensor per pass

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

// Tile `tile` of the gather's flat work list: rows of one module copied verbatim, plus their position IDs.
__device__ __forceinline__ void gather_tile(const GatherArgs &a, int tile, uint8_t *__restrict__ out_k,
                                            uint8_t *__restrict__ out_v, int32_t *__restrict__ out_pos)
{
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

    for (int base = 0; base < n_vec; base += kThreads * kUnroll) {
        u32x4 rk[kUnroll], rv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int i = base + u * kThreads + threadIdx.x;
            if (i < n_vec) {
                rk[u] = __builtin_nontemporal_load(sk + i);
                rv[u] = __builtin_nontemporal_load(sv + i);
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int i = base + u * kThreads + threadIdx.x;
            if (i < n_vec) {
                dk[i] = rk[u];
                dv[i] = rv[u];
            }
        }
    }
    for (int r = threadIdx.x; r < n_rows; r += kThreads)
        out_pos[sg.dst_row + r0 + r] = sg.start_pos + r0 + r;
}

// Row `row` of the append's flat work list, handled by one workgroup: K_new rotated at the row's
// position ID into the tail of the assembled K, V_new copied, the position ID written.
template <typename T>
__device__ __forceinline__ void append_row(const AppendSeg *seg, int n_segs, int row, const T *k_new, const T *v_new,
                                              const int32_t *q_pos, T *asm_k, T *asm_v, int32_t *asm_pos,
                                              int n_kv_heads, int d, const float2 *table, int max_pos)
{
    int r = row, s = 0;
    while (s < n_segs && r >= seg[s].n) {
        r -= seg[s].n;
        ++s;
    }
    if (s >= n_segs) return;
    const int src = seg[s].q_begin + r;
    const int dst = seg[s].dst_row + r;
    const int half = d >> 1;
    const int row_elems = n_kv_heads * d;
    const int p = q_pos[src];
    const float2 *trow = table + (size_t)clamp_pos(p, max_pos) * half;
    const T *ks = k_new + (size_t)src * row_elems;
    const T *vs = v_new + (size_t)src * row_elems;
    T *kd = asm_k + (size_t)dst * row_elems;
    T *vd = asm_v + (size_t)dst * row_elems;
    for (int e = threadIdx.x; e < n_kv_heads * half; e += kThreads) {
        const int h = e / half, i = e % half;
        const float2 cs = trow[i];
        const float lo = Elem<T>::load(ks + h * d + i), hi = Elem<T>::load(ks + h * d + i + half);
        Elem<T>::store(kd + h * d + i, lo * cs.x - hi * cs.y);
        Elem<T>::store(kd + h * d + i + half, hi * cs.x + lo * cs.y);
    }
    for (int e = threadIdx.x; e < row_elems; e += kThreads) vd[e] = vs[e];
    if (threadIdx.x == 0) asm_pos[dst] = p;
}

}  // namespace kv
}  // namespace pc
