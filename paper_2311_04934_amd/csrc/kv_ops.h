// Device bodies of the KV assembly: the gather of one tile of module rows and the append of one
// uncached token's row.  Shared by the stand-alone kernels and the fused assemble+append kernel.
#pragma once
#include "common.h"

namespace pc {
namespace kv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;
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

// Segment that holds `tile` of the gather's flat work list: the last one whose first_tile <= tile (uniform
// across the workgroup).
__device__ __forceinline__ int gather_segment(const GatherArgs &a, int tile)
{
    int lo = 0, hi = a.n_segs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (a.seg[mid].first_tile <= tile) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

__device__ __forceinline__ void gather_tile_of(const GatherArgs &a, const GatherSeg &sg, int tile, uint8_t *__restrict__ out_k,
                                               uint8_t *__restrict__ out_v, int32_t *__restrict__ out_pos);

// The head of a gather's arguments once more, as 14 dwords at the front of the kernel's argument list: one scalar
// load brings them all, and a launch of up to kHeadSegs segments then finds a tile's segment by comparisons, where the
// search over the table costs one dependent scalar load per step before the workgroup's first vector load can go
// out (12 segments: four).
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
constexpr int kHeadSegs = 12;
struct GatherHead {   // passed as ft[0], ft[1], ft[2], n: 14 dwords without padding
    i32x4 ft[3];    // first_tile of segments 0..11 (INT_MAX beyond n_segs)
    i32x2 n;        // n_segs, total_tiles
};
inline GatherHead gather_head(const GatherArgs &a)
{
    GatherHead h;
    h.n = i32x2{a.n_segs, a.total_tiles};
    for (int i = 0; i < kHeadSegs; ++i) h.ft[i >> 2][i & 3] = i < a.n_segs ? a.seg[i].first_tile : 0x7fffffff;
    return h;
}
__device__ __forceinline__ int gather_segment(const GatherArgs &a, i32x2 n, i32x4 f0, i32x4 f1, i32x4 f2, int tile)
{
    if (n[0] > kHeadSegs) return gather_segment(a, tile);
    int si = -1;   // segments whose first tile is <= tile, minus one (first_tile is ascending, INT_MAX past the end)
#pragma unroll
    for (int i = 0; i < 4; ++i) si += (f0[i] <= tile) + (f1[i] <= tile) + (f2[i] <= tile);
    return si;
}

// Tile `tile` of the gather's flat work list: rows of one module copied verbatim, plus their position IDs.
__device__ __forceinline__ void gather_tile(const GatherArgs &a, int tile, uint8_t *__restrict__ out_k,
                                            uint8_t *__restrict__ out_v, int32_t *__restrict__ out_pos)
{
    const GatherSeg sg = a.seg[gather_segment(a, tile)];
    gather_tile_of(a, sg, tile, out_k, out_v, out_pos);
}

__device__ __forceinline__ void gather_tile_of(const GatherArgs &a, const GatherSeg &sg, int tile, uint8_t *__restrict__ out_k,
                                               uint8_t *__restrict__ out_v, int32_t *__restrict__ out_pos)
{
    if (sg.src_k == nullptr) {   // rows copied by the copy engine: position IDs only, in larger tiles
        const int rpt = a.rows_per_tile * kPosOnlyTileFactor;
        const int p0 = (tile - sg.first_tile) * rpt;
        const int pn = sg.n_rows - p0 < rpt ? sg.n_rows - p0 : rpt;
        for (int r = threadIdx.x; r < pn; r += kThreads) out_pos[sg.dst_row + p0 + r] = sg.start_pos + p0 + r;
        return;
    }
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

// Eight consecutive elements of a row as floats (bf16: one 16-byte access; fp32: two).
template <typename T>
struct Vec8;
template <>
struct Vec8<uint16_t> {
    static __device__ __forceinline__ void load(const uint16_t *p, float (&x)[8])
    {
        const u32x4 w = *reinterpret_cast<const u32x4 *>(p);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = __uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16));
    }
    static __device__ __forceinline__ void store(uint16_t *p, const float (&x)[8])
    {
        typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
        bf16x8 w;
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = (__bf16)x[e];
        *reinterpret_cast<bf16x8 *>(p) = w;
    }
};
template <>
struct Vec8<float> {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ void load(const float *p, float (&x)[8])
    {
        const f32x4 a = *reinterpret_cast<const f32x4 *>(p), b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { x[e] = a[e]; x[4 + e] = b[e]; }
    }
    static __device__ __forceinline__ void store(float *p, const float (&x)[8])
    {
        f32x4 a, b;
#pragma unroll
        for (int e = 0; e < 4; ++e) { a[e] = x[e]; b[e] = x[4 + e]; }
        *reinterpret_cast<f32x4 *>(p) = a;
        *reinterpret_cast<f32x4 *>(p + 4) = b;
    }
};

// dst = rotation of src at one position (table row trow; nullptr: no rotation), times scale: n_heads heads of d
// elements, half-split pairs (element i with element i + d/2).  Run by a whole workgroup; a thread handles
// 8 pairs per pass when d is a multiple of 16.
template <typename T>
__device__ __forceinline__ void rotate_row(const T *__restrict__ src, T *__restrict__ dst, int n_heads, int d,
                                           const float2 *__restrict__ trow, float scale)
{
    const int half = d >> 1;
    if (d & 15) {   // odd head sizes (fp32 only): element by element
        for (int e = threadIdx.x; e < n_heads * half; e += kThreads) {
            const int h = e / half, i = e % half;
            const float2 cs = trow ? trow[i] : make_float2(1.f, 0.f);
            const float lo = Elem<T>::load(src + h * d + i), hi = Elem<T>::load(src + h * d + i + half);
            Elem<T>::store(dst + h * d + i, (lo * cs.x - hi * cs.y) * scale);
            Elem<T>::store(dst + h * d + i + half, (hi * cs.x + lo * cs.y) * scale);
        }
        return;
    }
    const int blocks_per_head = half >> 3;
    for (int blk = threadIdx.x; blk < n_heads * blocks_per_head; blk += kThreads) {
        const int h = blk / blocks_per_head, i0 = (blk % blocks_per_head) << 3;
        float lo[8], hi[8], olo[8], ohi[8];
        Vec8<T>::load(src + h * d + i0, lo);
        Vec8<T>::load(src + h * d + i0 + half, hi);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float2 cs = trow ? trow[i0 + e] : make_float2(1.f, 0.f);
            olo[e] = (lo[e] * cs.x - hi[e] * cs.y) * scale;
            ohi[e] = (hi[e] * cs.x + lo[e] * cs.y) * scale;
        }
        Vec8<T>::store(dst + h * d + i0, olo);
        Vec8<T>::store(dst + h * d + i0 + half, ohi);
    }
}

// Optional second job of an append row: the same token's query row, rotated at the same position and
// scaled, for attention calls that take Q already rotated.
template <typename T>
struct QRotate {
    const T *__restrict__ q_new = nullptr;   // [rows][n_q_heads][d], nullptr: nothing to do
    T *__restrict__ q_rot = nullptr;
    int n_q_heads = 0;
    float scale = 1.f;
};

// Row `row` of the append's flat work list, handled by one workgroup: K_new rotated at the row's
// position ID into the tail of the assembled K (copied as it is when table == nullptr: models with a
// linear attention bias, Sec. 4.2), V_new copied, the position ID written.
template <typename T>
__device__ __forceinline__ void append_row(const AppendSeg *seg, int n_segs, int row, const T *__restrict__ k_new,
                                           const T *__restrict__ v_new, const int32_t *__restrict__ q_pos,
                                           T *__restrict__ asm_k, T *__restrict__ asm_v, int32_t *__restrict__ asm_pos,
                                           int n_kv_heads, int d, const float2 *__restrict__ table, int max_pos,
                                           const QRotate<T> qr = QRotate<T>())
{
    int r = row, s = 0;
    while (s < n_segs && r >= seg[s].n) {
        r -= seg[s].n;
        ++s;
    }
    if (s >= n_segs) return;
    const int src = seg[s].q_begin + r;
    const int dst = seg[s].dst_row + r;
    const int mode = seg[s].pos0;
    if (mode == kPosMaskRows) {   // an unused placeholder row: it stops being a token, its states stay
        if (threadIdx.x == 0) asm_pos[dst] = PC_POS_NONE;
        return;
    }
    const int half = d >> 1;
    const int row_elems = n_kv_heads * d;
    const int p = mode >= 0 ? mode + r : q_pos[src];
    const float2 *trow = table ? table + (size_t)clamp_pos(p, max_pos) * half : nullptr;
    const T *ks = k_new + (size_t)src * row_elems;
    const T *vs = v_new + (size_t)src * row_elems;
    T *kd = asm_k + (size_t)dst * row_elems;
    T *vd = asm_v + (size_t)dst * row_elems;
    // V (and K when it is not rotated) first: these copies do not depend on the position ID
    if ((row_elems * sizeof(T)) & 15) {
        for (int e = threadIdx.x; e < row_elems; e += kThreads) {
            vd[e] = vs[e];
            if (!trow) kd[e] = ks[e];
        }
    } else {
        const int n_vec = (int)((size_t)row_elems * sizeof(T) >> 4);
        for (int i = threadIdx.x; i < n_vec; i += kThreads) {
            reinterpret_cast<u32x4 *>(vd)[i] = reinterpret_cast<const u32x4 *>(vs)[i];
            if (!trow) reinterpret_cast<u32x4 *>(kd)[i] = reinterpret_cast<const u32x4 *>(ks)[i];
        }
    }
    if (qr.q_new) {
        const size_t q_elems = (size_t)qr.n_q_heads * d;
        rotate_row<T>(qr.q_new + (size_t)src * q_elems, qr.q_rot + (size_t)src * q_elems, qr.n_q_heads, d, trow, qr.scale);
    }
    if (trow) rotate_row<T>(ks, kd, n_kv_heads, d, trow, 1.f);
    if (threadIdx.x == 0) asm_pos[dst] = p;
}

}  // namespace kv
}  // namespace pc
