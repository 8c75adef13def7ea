// Uncached-token prefill attention over the assembled KV (Sec. 3.4 of the paper), bf16 MFMA,
// head_dim 128: 8 wavefronts per workgroup (two per SIMD), one 32-query row tile per wavefront.
//
// Same contract and the same S^T = K.Q^T / O^T += V^T.P^T formulation as the register-staged
// kernel (attn_bf16.hip); what differs is how the work is fed:
//
//   staging   K, V and position IDs of a 64-key tile go from global memory straight into LDS
//             (global_load_lds, 16 bytes per lane): no registers, no LDS-write instructions.
//             The copies of tile T+3 are issued while tile T is computed.  Rows are stored
//             unpadded with their 16-byte chunks XOR-swizzled by the key index so that both the
//             K reads (one key per lane) and the transposing V reads are bank-conflict free.
//             Over the packed buffer a copy instruction takes a wave-uniform base address (the
//             tile's first row, advanced from tile to tile) and a per-lane offset that never changes.
//   V         lands row-major [key][d].  Once per tile the workgroup re-lays it out as MFMA A
//             fragments of V^T: each wave fetches two of the 16 fragments with ds_read_b64_tr_b16
//             and stores them lane-major, so that all 8 waves then read a fragment with a single
//             16-byte LDS load.
//   pipeline  a step handles three independent pieces of work on three 32-key sub-tiles: P.V of
//             the previous one, K.Q of the next one and the online softmax of the current one.
//             Matrix and vector instructions of the same wave overlap when they alternate, so a
//             step is written as 16 slots of one matrix instruction followed by one softmax
//             element (see step()).  The copies of the next tile and the V re-layout ride in
//             the same slots.  One workgroup barrier per 64-key tile.
//   rescale   O is rescaled only when the reference maximum of the online softmax moved, which
//             it does rarely: the reference follows the running maximum lazily (see kMaxSlack).
//   mask      by position ID (visible iff pos_k <= pos_q).  Per wave and tile a vote on the tile's
//             position IDs decides: every key visible (no mask), some (per-element compare), none:
//             the wave then skips the tile's arithmetic altogether and only does its share of the
//             staging (uncached text placed before later modules, Sec. 3.4; ordinary causal prefill;
//             packed buffer only).
//   epilogue  the two lanes that hold a query exchange halves of their accumulators, after which
//             each owns 16 consecutive d of the row: the output (or, split over the keys, the
//             un-normalised partial O in bf16 and (m, l)) goes out in 16-byte stores, without LDS
//             or a barrier.
//
// The kernel is a template over the number of row tiles per wave; only <1 tile, 8 waves> is
// instantiated (two tiles per wave need all 512 registers, which leaves one wave per SIMD, and
// measured slower).

#include <type_traits>

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
constexpr int NVRAW = 3;                         // landing buffers of V as it is in global memory
constexpr int NVT = 2;                           // buffers of V re-laid out as MFMA fragments
constexpr int LDS_K = 0;
constexpr int LDS_V = NBUF * TILE_BYTES;                     // 64 KiB: raw V, [key][d], swizzled chunks
constexpr int LDS_VT = LDS_V + NVRAW * TILE_BYTES;           // 112 KiB: V^T fragments, 16 x 1 KiB per tile
constexpr int LDS_POS = LDS_VT + NVT * TILE_BYTES;           // 144 KiB
constexpr int LDS_BIAS = LDS_POS + NBUF * KT * 4;          // linear-bias variant: per wave, 2 tiles x 64 floats
constexpr int LDS_MAIN = LDS_BIAS + kWideRowTilesPerWg * 2 * KT * 4;
constexpr int LDS_TOTAL = LDS_MAIN;

typedef __attribute__((address_space(3))) uint8_t lds_u8;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// s_waitcnt that only waits for the vector-memory counter to drop to n (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "don't wait").
#define PC_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))
// the same, and the LDS/scalar-memory counter down to m (no scalar loads may be in flight: they return out of order)
#define PC_WAIT_VM_LGKM(n, m) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | ((m) << 8))

// Asynchronous global -> LDS copy of 16 (or 4) bytes per lane: lane l's data lands at
// lds_addr + 16*l (4*l).  Issued as inline assembly so that the compiler does not make every
// later LDS read wait for it; completion is awaited explicitly with PC_WAIT_VMCNT before the
// workgroup barrier that publishes a tile.  Two address forms: a full 64-bit address per lane,
// or a wave-uniform 64-bit base (scalar registers) plus a 32-bit offset per lane.
__device__ __forceinline__ void dma_b128(const void *gsrc, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gsrc) : "memory", "m0");
}
__device__ __forceinline__ void dma_b32(const void *gsrc, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(gsrc) : "memory", "m0");
}
// the value is the same in every lane: tells the compiler so (scalar registers)
__device__ __forceinline__ uint64_t uniform_u64(uint64_t x)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x), hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ void dma_b128_u(uint64_t base, uint32_t lane_off, uint32_t lds_addr)
{
    base = uniform_u64(base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}
__device__ __forceinline__ void dma_b32_u(uint64_t base, uint32_t lane_off, uint32_t lds_addr)
{
    base = uniform_u64(base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}

// Row tile rt of a kv head's stack (query heads of the group one after the other, tiles_q tiles each): which head of the
// group and which tile of the prompt's queries.  rt is wave-uniform and groups are small: a few scalar subtractions
// instead of a division.
__device__ __forceinline__ void split_row_tile(int rt, int tiles_q, int G, int &g_head, int &tq)
{
    if (G <= 8) {
        g_head = 0;
        tq = rt;
        while (tq >= tiles_q) {
            tq -= tiles_q;
            ++g_head;
        }
    } else {
        g_head = rt / tiles_q;
        tq = rt - g_head * tiles_q;
    }
}

struct QTile {        // one 32-query row tile of a wave
    bool valid;       // this lane's query exists
    int head;
    int tq;           // index of the 32-query tile inside the prompt
    int qi;           // query index inside the prompt
    int qpos;         // its position ID (+inf when the lane has no query)
};

struct NoSegTable {
    int unused;
};

// PAGED: the keys come from a list of row ranges (see KvSegTable) instead of one packed buffer.
// ALIBI: position enters as the linear bias -slope[head] * (pos_q - pos_k) on the scores (Sec. 4.2 of the
// paper: the bias follows the given position IDs) instead of a rotation of Q; keys are stored unrotated.
template <int NQT, int NW, bool PAGED, bool ALIBI>
__global__ __launch_bounds__(NW * 64) void attn_bf16_dma_kernel(const i32x4 h0, const i32x4 h1, const i32x4 h2, const i32x2 h3,
                                                                const AttnParams p,
                                                                const std::conditional_t<PAGED, KvSegTable, NoSegTable> tab)
{
    // What the first copies of the kernel depend on (which work unit, which rows, which keys, where K, V and the
    // position IDs are) comes a second time as the first 14 dwords of the argument list, which the dispatcher puts
    // into scalar registers before the wave starts (the build asks for that): the first K/V tile is requested
    // without a trip to the argument buffer (measured: ~1000 cycles per dependent round of scalar loads at the start
    // of a kernel), and the loads of everything else, issued at once, arrive behind it.  See attn_head() for the packing.
    const int a_hkv_shift = h0[0], a_share0 = h0[1];   // log2 of the kv heads padded to a power of two; first prompt's keys per split
    const int a_Hkv = h0[2] & 0xff, a_n_splits = (h0[2] >> 8) & 0xff, a_G = (h0[2] >> 16) & 0xff, a_q_rotated = (h0[2] >> 24) & 1;
    const int a_n_seqs = h0[3] & 0xff, a_Hq = (int)((unsigned)h0[3] >> 8);
    const AttnSeq a_seq0 = {h1[0], h1[1], h1[2], h1[3]};
    const uint16_t *const a_k = reinterpret_cast<const uint16_t *>(((uint64_t)(uint32_t)h2[1] << 32) | (uint32_t)h2[0]);
    const uint16_t *const a_v = reinterpret_cast<const uint16_t *>(((uint64_t)(uint32_t)h2[3] << 32) | (uint32_t)h2[2]);
    const int32_t *const a_kv_pos = reinterpret_cast<const int32_t *>(((uint64_t)(uint32_t)h3[1] << 32) | (uint32_t)h3[0]);
    static_assert(NQT * NW == kWideRowTilesPerWg, "a workgroup covers 8 row tiles");
    static_assert(NQT == 1, "one row tile per wave (the softmax state below is kept per wave)");
    constexpr int GRP_PER_WAVE = 16 / NW;                // 1-KiB (4-row) groups of a tile each wave copies, per tensor
    constexpr int DMA_PER_TILE = 2 * GRP_PER_WAVE + 1;   // loads a wave issues per tile (K, V, positions)

    extern __shared__ __align__(16) uint8_t smem[];
    lds_u8 *lds = (lds_u8 *)smem;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: lives in a scalar register
    const int wave_s = wave;
    const int col = lane & 31;
    const int hh = lane >> 5;

    // ---- work unit.  The grid is (kv heads padded to a power of two x row blocks, KV splits, prompts): no division
    // stands between the wave's start and its first copy.  Workgroups are dealt to the 8 XCDs in the order of their
    // linear index, x fastest, so with the kv head fastest the XCD follows the kv head (8 or more of them): all KV
    // splits of a (prompt, kv head) run on one XCD and fetch the query rows of that head group once into its L2
    // (with the split fastest, every XCD fetched the whole Q: 8 x 2.1 MB at config 3), while each K/V range is
    // still read by one XCD only.
    const int kvh = blockIdx.x & ((1 << a_hkv_shift) - 1);
    const int rb = blockIdx.x >> a_hkv_shift;
    const int split = blockIdx.y;
    const int seq_i = blockIdx.z;
    if (kvh >= a_Hkv) return;
    AttnSeq seq = a_seq0;
    if (a_n_seqs > 1) seq = p.batch.seq[seq_i];

    const int tiles_q = (seq.n_q + RW - 1) / RW;
    const int row_tiles = a_G * tiles_q;
    if (rb * kWideRowTilesPerWg >= row_tiles) return;

    // a split's share of the keys is a whole number of 64-key tiles: only the last split of a prompt then ends in a
    // ragged tile (which costs a masked iteration), and with 16.5 tiles per split every split would have one
    const int share = a_n_seqs > 1 ? (((seq.n_kv + a_n_splits - 1) / a_n_splits) + KT - 1) & ~(KT - 1) : a_share0;
    const int k_begin = split * share < seq.n_kv ? split * share : seq.n_kv;
    const int k_end = k_begin + share < seq.n_kv ? k_begin + share : seq.n_kv;
    const int n_tiles = (k_end - k_begin + KT - 1) / KT;

    // Without a rotation to look up (Q arrives rotated, or position enters as a linear bias) nothing depends on the
    // queries' position IDs before the first mask decision: they then travel with the asynchronous copies instead
    // of holding these up (uniform)
    const bool q_rot = a_q_rotated != 0;   // Q was rotated and scaled by the caller (append/assemble call)
    const bool q_direct = ALIBI || q_rot;

    // ---- this wave's row tile
    QTile qt[NQT];
#pragma unroll
    for (int x = 0; x < NQT; ++x) {
        const int rt = rb * kWideRowTilesPerWg + wave * NQT + x;
        const bool act = rt < row_tiles;
        int g_head = 0, tq = 0;
        if (act) split_row_tile(rt, tiles_q, a_G, g_head, tq);
        qt[x].head = kvh * a_G + g_head;
        qt[x].tq = tq;
        qt[x].qi = tq * RW + col;
        qt[x].valid = act && qt[x].qi < seq.n_q;
        qt[x].qpos = (qt[x].valid && !q_direct) ? p.q_pos[seq.q_begin + qt[x].qi] : kPosInf;
    }

    // ALIBI: this wave's slope in the log2 domain.  The head is the same for the wave's 32 queries, so the
    // load is a scalar one (it does not touch the vector-memory counter the copies are tracked with).
    float slope2 = 0.f;
    if constexpr (ALIBI) slope2 = p.alibi[__builtin_amdgcn_readfirstlane(qt[0].head)] * 1.4426950408889634f;

    const size_t kv_row_stride = (size_t)a_Hkv * D;  // elements
    const uint16_t *k_base = PAGED ? nullptr : a_k + (size_t)seq.kv_begin * kv_row_stride + (size_t)kvh * D;
    const uint16_t *v_base = PAGED ? nullptr : a_v + (size_t)seq.kv_begin * kv_row_stride + (size_t)kvh * D;
    const int32_t *pos_base = PAGED ? nullptr : a_kv_pos + seq.kv_begin;
    const int last_row = k_end - 1;

    // PAGED: which row range holds a given row of the prompt.  The range table stays in the kernel
    // arguments and is only ever indexed with wave-uniform values, i.e. through the scalar cache: a
    // vector-memory load between the asynchronous copies would have to wait for all of them.  Tiles
    // are requested in increasing order, so the wave keeps the range of the tile's first row in scalar
    // registers (seg_cur, its pointers, its first row and the next range's first row): a tile inside
    // one range, the usual case, is copied from a uniform base like a tile of the packed buffer.  Only a
    // tile that straddles a boundary walks the ranges it touches and selects per lane.
    int seg_cur = 0, seg_lo = 0, n_seg = 0;
    uint32_t cur_first = 0, next_first = 0xffffffffu;
    uint64_t cur_k = 0, cur_v = 0, cur_p = 0;
    auto seg_at = [&](int e) -> KvSeg {   // e uniform, < n_seg
        if constexpr (PAGED) return tab.seg[__builtin_amdgcn_readfirstlane(seg_lo + e)];
        else return KvSeg{};
    };
    auto uniform64 = [](uint64_t x) -> uint64_t {   // tells the compiler that the value is the same in every lane
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x), hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
        return ((uint64_t)hi << 32) | lo;
    };
    auto load_seg = [&](int e) {
        const KvSeg sg = seg_at(e);
        cur_k = uniform64(reinterpret_cast<uint64_t>(sg.k));
        cur_v = uniform64(reinterpret_cast<uint64_t>(sg.v));
        cur_p = uniform64(reinterpret_cast<uint64_t>(sg.pos));
        cur_first = __builtin_amdgcn_readfirstlane((uint32_t)sg.first_row);
        next_first = e + 1 < n_seg ? __builtin_amdgcn_readfirstlane((uint32_t)seg_at(e + 1).first_row) : 0xffffffffu;
    };
    if constexpr (PAGED) {
        seg_lo = tab.seg_begin[seq_i];
        n_seg = tab.seg_begin[seq_i + 1] - seg_lo;
        load_seg(0);   // a prompt with query rows has at least the range of its own tokens
    }
    auto advance_to = [&](uint32_t row) {   // uniform row: first row the coming requests can touch
        if constexpr (PAGED)
            while (next_first <= row) {
                seg_cur = __builtin_amdgcn_readfirstlane(seg_cur + 1);
                load_seg(seg_cur);
            }
    };
    // row (per lane, >= the row of the last advance_to, < row_hi) -> the addresses of that row's K, V and position
    auto locate = [&](uint32_t row, uint32_t row_hi, const uint8_t *&kp, const uint8_t *&vp, const int32_t *&pp) {
        if constexpr (PAGED) {
            const uint32_t head_off = (uint32_t)(kvh * D * 2), stride = (uint32_t)(kv_row_stride * 2u);
            uint64_t bk = cur_k, bv = cur_v, bp = cur_p;
            uint32_t first = cur_first;
            if (next_first < row_hi) {   // uniform: the tile runs into later ranges
                for (int sx = seg_cur + 1; sx < n_seg; ++sx) {
                    const KvSeg sg = seg_at(sx);
                    if ((uint32_t)sg.first_row >= row_hi) break;
                    const bool in = row >= (uint32_t)sg.first_row;
                    bk = in ? reinterpret_cast<uint64_t>(sg.k) : bk;
                    bv = in ? reinterpret_cast<uint64_t>(sg.v) : bv;
                    bp = in ? reinterpret_cast<uint64_t>(sg.pos) : bp;
                    first = in ? (uint32_t)sg.first_row : first;
                }
            }
            const uint32_t local = row - first;
            const uint32_t off = local * stride + head_off;   // < 4 GiB per range
            kp = reinterpret_cast<const uint8_t *>(bk) + off;
            vp = reinterpret_cast<const uint8_t *>(bv) + off;
            pp = reinterpret_cast<const int32_t *>(bp) + local;
        }
    };

    // ---- global -> LDS, asynchronously.  One wave instruction fills 1 KiB = 4 rows; LDS slot
    // (row r, 16-byte chunk c) receives global chunk c ^ swz(r).  A wave issues exactly DMA_PER_TILE loads per
    // tile: group j of its K rows, group j of its V rows (j < GRP_PER_WAVE), then the 64 position IDs.  Tiles are
    // issued strictly in order, each exactly once: begin_tile(t), then its pieces.
    // Rows past the split's end are read from its last row (finite values; they are masked by index in the
    // softmax), and a tile past the end lands in a buffer nobody reads again, which keeps the count of
    // outstanding copies the same in every iteration.
    //
    // Packed buffer: a copy takes a wave-uniform base in scalar registers, the address of the tile's first row,
    // which simply advances from tile to tile, and a 32-bit offset per lane that never changes (the lane's row of
    // the tile times the row pitch, plus its swizzled chunk): a tile costs a few scalar instructions.  Only a
    // tile that is not whole (the ragged end of a prompt, the look-ahead past the end) clamps rows per lane; that
    // is done apart from the hand-scheduled step.  PAGED: every lane forms its own 64-bit address.
    const uint32_t row_bytes_g = (uint32_t)kv_row_stride * 2u;   // bytes between consecutive keys in global memory
    const uint8_t *k_bytes = reinterpret_cast<const uint8_t *>(k_base);
    const uint8_t *v_bytes = reinterpret_cast<const uint8_t *>(v_base);
    static_assert(NW == 8 && GRP_PER_WAVE == 2, "group 1 of a wave's rows is 32 rows below group 0: the swizzles of both groups agree");
    const uint32_t dma_r0 = (uint32_t)(wave * 4 + (lane >> 4));                         // this lane's row of the tile in group 0
    const uint32_t dma_ck = (uint32_t)(((lane & 15) ^ (int)(dma_r0 & 15)) << 4);        // byte offset of its chunk inside a K row
    const uint32_t dma_cv = (uint32_t)(((lane & 15) ^ (int)((dma_r0 & 7) << 1)) << 4);  // ... inside a V row
    const uint32_t off_k0 = PAGED ? 0u : dma_r0 * row_bytes_g + dma_ck;   // group 0 of a whole tile (group 1: 32 rows further)
    const uint32_t off_v0 = PAGED ? 0u : dma_r0 * row_bytes_g + dma_cv;
    const uint32_t off_p = (uint32_t)lane * 4u;
    const uint32_t grp_step = 32u * row_bytes_g;
    const uint32_t dst_wave = lds_base + (uint32_t)wave_s * 1024u;
    // state of the tile whose pieces are being issued (wave-uniform, set by begin_tile)
    uint64_t run_k = PAGED ? 0 : uniform_u64(reinterpret_cast<uint64_t>(k_bytes) + (uint64_t)k_begin * row_bytes_g);
    uint64_t run_v = PAGED ? 0 : uniform_u64(reinterpret_cast<uint64_t>(v_bytes) + (uint64_t)k_begin * row_bytes_g);
    uint64_t run_p = PAGED ? 0 : uniform_u64(reinterpret_cast<uint64_t>(pos_base + k_begin));
    int run_row = k_begin, run_vraw = 0;   // first row of the next tile to issue, and its raw-V buffer (tile index mod NVRAW)
    uint64_t tile_k = 0, tile_v = 0, tile_p = 0;
    uint32_t dst_k = 0, dst_v = 0, dst_p = 0;
    // returns whether tile t is whole (its pieces then go out through whole_piece, else through ragged_tile)
    auto begin_tile = [&](int t) -> bool {
        const int buf = t & (NBUF - 1);
        dst_k = dst_wave + LDS_K + (uint32_t)buf * TILE_BYTES;
        dst_v = dst_wave + LDS_V + (uint32_t)run_vraw * TILE_BYTES;
        dst_p = lds_base + LDS_POS + (uint32_t)buf * KT * 4;
        run_vraw = run_vraw == NVRAW - 1 ? 0 : run_vraw + 1;
        if constexpr (PAGED) {
            const uint32_t row0 = (uint32_t)(k_begin + t * KT);
            advance_to(row0 < (uint32_t)last_row ? row0 : (uint32_t)last_row);
            return true;
        } else {
            const bool whole = run_row + KT <= k_end;
            tile_k = run_k;
            tile_v = run_v;
            tile_p = run_p;
            run_k += (uint64_t)KT * row_bytes_g;   // not used any more once a tile was not whole (no later one is)
            run_v += (uint64_t)KT * row_bytes_g;
            run_p += (uint64_t)KT * 4u;
            run_row += KT;
            return whole;
        }
    };
    // piece k of a whole tile (PAGED: of any tile): k < 2*GRP_PER_WAVE is a K (even) or V (odd) group, the last
    // piece is the position IDs
    auto whole_piece = [&](int t, int k) {
        if (k < 2 * GRP_PER_WAVE) {
            const int j = k >> 1;
            const uint32_t dst = ((k & 1) ? dst_v : dst_k) + (uint32_t)(j * NW) * 1024u;
            if constexpr (PAGED) {
                const uint32_t row0 = (uint32_t)(k_begin + t * KT);
                const uint32_t row_hi = row0 + KT < (uint32_t)k_end ? row0 + KT : (uint32_t)k_end;
                uint32_t grow = row0 + dma_r0 + (uint32_t)(j * NW * 4);
                grow = grow < (uint32_t)last_row ? grow : (uint32_t)last_row;
                const uint8_t *kp, *vp;
                const int32_t *pp;
                locate(grow, row_hi, kp, vp, pp);
                if (k & 1) dma_b128(vp + dma_cv, dst);
                else dma_b128(kp + dma_ck, dst);
            } else {
                const uint32_t voff = ((k & 1) ? off_v0 : off_k0) + (j ? grp_step : 0u);
                dma_b128_u((k & 1) ? tile_v : tile_k, voff, dst);
            }
        } else {
            if constexpr (PAGED) {
                const uint32_t row0 = (uint32_t)(k_begin + t * KT);
                const uint32_t row_hi = row0 + KT < (uint32_t)k_end ? row0 + KT : (uint32_t)k_end;
                uint32_t prow = row0 + (uint32_t)lane;
                prow = prow < (uint32_t)last_row ? prow : (uint32_t)last_row;
                const uint8_t *kp, *vp;
                const int32_t *pp;
                locate(prow, row_hi, kp, vp, pp);
                dma_b32(pp, dst_p);
            } else {
                dma_b32_u(tile_p, off_p, dst_p);
            }
        }
    };
    // all pieces of a tile of the packed buffer that is not whole: rows clamped per lane to the split's last row
    auto ragged_tile = [&](int t) {
        if constexpr (!PAGED) {
            const int lane_x = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
            const uint32_t row0 = (uint32_t)(k_begin + t * KT);
#pragma unroll
            for (int k = 0; k < 2 * GRP_PER_WAVE; ++k) {
                const int j = k >> 1;
                const uint32_t r = (uint32_t)((j * NW + wave_s) * 4 + (lane_x >> 4)), c = (uint32_t)(lane_x & 15);
                uint32_t grow = row0 + r;
                grow = grow < (uint32_t)last_row ? grow : (uint32_t)last_row;
                const uint32_t chunk = (k & 1) ? ((c ^ ((r & 7) << 1)) << 4) : ((c ^ (r & 15)) << 4);
                const uint32_t off = grow * row_bytes_g + chunk;               // < 4 GiB, checked by the launcher
                dma_b128(((k & 1) ? v_bytes : k_bytes) + off, ((k & 1) ? dst_v : dst_k) + (uint32_t)(j * NW) * 1024u);
            }
            uint32_t prow = row0 + (uint32_t)lane_x;
            prow = prow < (uint32_t)last_row ? prow : (uint32_t)last_row;
            dma_b32(pos_base + prow, dst_p);
        }
    };
    auto issue_tile = [&](int t) {
        if (begin_tile(t)) {
#pragma unroll
            for (int k = 0; k < DMA_PER_TILE; ++k) whole_piece(t, k);
        } else {
            ragged_tile(t);
        }
    };

    // ---- prologue.  Order matters for latency.  When Q has to be rotated here, the position IDs come first
    // (the rotation-table addresses depend on them), then three kinds of requests go out together: the first
    // two K/V tiles (from HBM, the longest wait, so they go first); the raw Q rows, as asynchronous copies into
    // LDS (whole 256-byte rows per 16 lanes, where a direct load into the MFMA operand layout would touch 32 cache
    // lines per instruction); and the table values.  The compiler does not see the copies: when it waits for the
    // table values, the older copies still in flight make that wait longer (all of them are needed now anyway),
    // while younger copies could let the count drop early, so the third tile is issued later.
    // When Q needs no table, everything is a copy, and copies complete in order: the position IDs, the first tile,
    // the Q rows, the second tile; only the second tile is not waited for before the first matrix instruction.
    //
    // Q staging space: row tile s = wave*NQT + x of the workgroup gets 8 KiB of tile buffers that stay
    // unused until the first workgroup barrier: K buffers 2 and 3, raw-V buffer 2, V^T buffer 1.
    auto q_region = [&](int s8) -> int {
        return s8 < 4 ? LDS_K + 2 * TILE_BYTES + s8 * 8192
                      : (s8 < 6 ? LDS_V + 2 * TILE_BYTES + (s8 - 4) * 8192 : LDS_VT + TILE_BYTES + (s8 - 6) * 8192);
    };
    static_assert(NVRAW == 3 && NVT == 2 && NBUF == 4 && NQT * NW == 8, "Q staging relies on this tile-buffer layout");
    bf16x8 qf[NQT][KB];
    auto copy_q_rows = [&]() {
#pragma unroll
        for (int x = 0; x < NQT; ++x) {
            const uint8_t *qhead = reinterpret_cast<const uint8_t *>(p.q) + ((size_t)seq.q_begin * a_Hq + qt[x].head) * (D * 2);
            const uint32_t dst0 = __builtin_amdgcn_readfirstlane(lds_base + q_region(wave * NQT + x));
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = 4 * j + (lane >> 4), c = lane & 15;   // row of the tile, 16-byte chunk of the row
                int qi = qt[x].tq * RW + r;
                qi = qi < seq.n_q ? qi : seq.n_q - 1;                // rows past the prompt's last query: any valid row
                dma_b128(qhead + (size_t)qi * a_Hq * (D * 2) + ((c ^ (r & 15)) << 4), dst0 + j * 1024);
            }
        }
    };
    if (n_tiles > 0) {
        float2 cs[NQT][KB / 2][8];
        if (q_direct) {
            // copies complete in the order they were issued: the queries' position IDs (one per lane, into this wave's
            // strip of the bias area, which nothing uses before the first mask decision), tile 0 and the Q rows are
            // waited for, tile 1 stays in flight until the loop's first barrier
            const int qi0 = qt[0].qi < seq.n_q ? qt[0].qi : seq.n_q - 1;
            issue_tile(0);   // needs nothing from the argument buffer
            dma_b32(p.q_pos + seq.q_begin + qi0, __builtin_amdgcn_readfirstlane(lds_base + LDS_BIAS + wave * 2 * KT * 4));
            copy_q_rows();
            issue_tile(1);
            PC_WAIT_VMCNT(DMA_PER_TILE);
            const int qp = *reinterpret_cast<const __attribute__((address_space(3))) int *>(lds + LDS_BIAS + wave * 2 * KT * 4 + lane * 4);
            qt[0].qpos = qt[0].valid ? qp : kPosInf;
        } else {
            int qq = qt[0].qpos;
            asm volatile("" : "+v"(qq));   // the position IDs have arrived
            qt[0].qpos = qq;
            // K/V come from HBM and are requested first; the Q rows (shared by all KV splits) mostly hit in cache
            issue_tile(0);
            issue_tile(1);
            copy_q_rows();
            // table values (position-minor table: the 32 lanes of a half-wave hold 32 queries, usually at
            // consecutive positions, so one pair index is a contiguous 256-byte read for them)
#pragma unroll
            for (int x = 0; x < NQT; ++x) {
                int tpos = qt[x].qpos;
                tpos = tpos < 0 ? 0 : (tpos >= p.max_pos ? p.max_pos - 1 : tpos);
                const float2 *tcol = p.rope_t + tpos;
#pragma unroll
                for (int kb = 0; kb < KB / 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 8; ++e) cs[x][kb][e] = tcol[(size_t)(kb * 16 + hh * 8 + e) * p.max_pos];
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // Q rows and tiles 0 and 1 have landed, the table values too
        }
        // Q rotated at the queries' position IDs, scaled by log2(e)/sqrt(d), bf16: B operand of K.Q
#pragma unroll
        for (int x = 0; x < NQT; ++x) {
            const lds_u8 *qrow = lds + q_region(wave * NQT + x) + col * ROW_BYTES;
#pragma unroll
            for (int kb = 0; kb < KB / 2; ++kb) {
                const u32x4 lo = *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(qrow + (((2 * kb + hh) ^ (col & 15)) << 4));
                const u32x4 hi = *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(qrow + (((2 * kb + hh + 8) ^ (col & 15)) << 4));
                if (q_rot) {   // the staged values are the operand
                    qf[x][kb] = __builtin_bit_cast(bf16x8, lo);
                    qf[x][kb + KB / 2] = __builtin_bit_cast(bf16x8, hi);
                    continue;
                }
                bf16x8 olo, ohi;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t wl = lo[e >> 1], wh = hi[e >> 1];
                    const float xl = bf16_bits_to_f32((e & 1) ? (wl >> 16) : (wl & 0xffffu));
                    const float xh = bf16_bits_to_f32((e & 1) ? (wh >> 16) : (wh & 0xffffu));
                    if constexpr (ALIBI) {   // Q as it is, scaled
                        olo[e] = (__bf16)(xl * p.q_scale);
                        ohi[e] = (__bf16)(xh * p.q_scale);
                    } else {
                        olo[e] = (__bf16)((xl * cs[x][kb][e].x - xh * cs[x][kb][e].y) * p.q_scale);
                        ohi[e] = (__bf16)((xh * cs[x][kb][e].x + xl * cs[x][kb][e].y) * p.q_scale);
                    }
                }
                qf[x][kb] = olo;
                qf[x][kb + KB / 2] = ohi;
            }
        }
    }
    // smallest query position in the wave: a key tile whose largest position exceeds it needs the mask;
    // largest one: a key tile whose smallest position exceeds it has nothing this wave can see
    const int wave_min_qpos = wave_min_i32(qt[0].qpos);
    const int wave_max_qpos = wave_max_i32(qt[0].valid ? qt[0].qpos : (int)0x80000000);
    const int bias_ref = wave_min_qpos;   // ALIBI: origin of the per-key bias (an idle wave's value is never used)

    // ---- per-lane LDS offsets of the MFMA operand fragments
    // K (A operand of K.Q): key = col of the sub-tile, chunk 2*kb+hh, swizzled by key & 15
    // (2 kb + hh) ^ (col & 15) = (hh ^ (col & 15)) ^ 2 kb: the eight offsets differ by an exclusive-or with kb << 5.
    // PAGED (which needs registers for its per-lane addresses) keeps one offset and applies that per read.
    constexpr int NKOFF = PAGED ? 1 : KB;
    int koff_r[NKOFF];
#pragma unroll
    for (int kb = 0; kb < NKOFF; ++kb) koff_r[kb] = col * ROW_BYTES + (((2 * kb + hh) ^ (col & 15)) << 4);
    auto koff = [&](int kb) -> int { return PAGED ? (koff_r[0] ^ (kb << 5)) : koff_r[PAGED ? 0 : kb]; };
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
    f32x16 o_acc[DB];
    float m_run = -INFINITY, l_run = 0.f, alpha = 1.f;   // running max / sum; alpha = pending rescale of O
    bool rescale_pending = false;   // wave-uniform: some lane's alpha differs from 1
    bf16x8 pf[2][2];                // [sub-tile parity][16-key half]
    f32x16 sc[2];                   // [sub-tile parity] scores
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[b][i] = 0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[a][j][e] = (__bf16)0.f;

    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
#define PC_FENCE() __builtin_amdgcn_sched_barrier(0)

    // V fragments (A operand of O^T += V^T.P^T) of one 32-key sub-tile, group g of 8 (two
    // transposing reads each): g = 4*j + b covers keys 16*j.., d rows 32*b..
    bf16x8 vf[2 * DB];
    auto read_v = [&](const lds_u8 *vbase, int g) {
        vf[g] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const lds_u32x4 *>(vbase + g * 1024 + lane * 16));
    };
    // Re-layout of V: fragment f = 8*sub + 4*j + b of a tile (keys 32*sub + 16*j .., d rows 32*b ..) is
    // fetched from the raw tile with two transposing reads, exactly the 16 bytes per lane the MFMA
    // wants, and stored lane-major, 1 KiB per fragment.  Each wave converts NW-th of the tile; all
    // waves then fetch a fragment with one 16-byte read instead of two transposing 8-byte ones.
    constexpr int FRAG_PER_WAVE = 16 / NW;
    s16x4 tr_lo[FRAG_PER_WAVE], tr_hi[FRAG_PER_WAVE];
    auto transpose_read = [&](int t, int k) {
        const int f = wave * FRAG_PER_WAVE + k;
        const int sub = f >> 3, j = (f >> 2) & 1, b = f & 3;
        const lds_u8 *a0 = lds + LDS_V + (t % NVRAW) * TILE_BYTES + (32 * sub + 16 * j) * ROW_BYTES + voff[b];
        tr_lo[k] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)a0);
        tr_hi[k] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0 + 8 * ROW_BYTES));
    };
    auto transpose_write = [&](int t, int k) {
        const int f = wave * FRAG_PER_WAVE + k;
        const s16x8 w = __builtin_shufflevector(tr_lo[k], tr_hi[k], 0, 1, 2, 3, 4, 5, 6, 7);
        *reinterpret_cast<__attribute__((address_space(3))) u32x4 *>(lds + LDS_VT + (t & (NVT - 1)) * TILE_BYTES + f * 1024 + lane * 16) = __builtin_bit_cast(u32x4, w);
    };

    // One step.  Three independent pieces of work on three different 32-key sub-tiles:
    //   O += V^T.P of the previous sub-tile (fragments vf were read during the previous step),
    //   S(next) = K.Q of the sub-tile after the current one,
    //   online softmax of the current scores s into pout (O is not rescaled here, see rescale()).
    // The code is laid out as 16 slots: one matrix instruction, then a share of the softmax's vector
    // instructions, one LDS read (slots 0..7: the K fragment that slot 8+i multiplies, into registers a V
    // fragment has just left; slots 8..15: the V fragments of the next step) and, when do_dma, one asynchronous
    // copy of that tile.  The compiler's scheduler is fenced between slots so that this order survives; the
    // empty asm statements keep each value's computation in its slot.
    auto step = [&](const bf16x8 (&pp)[2], const lds_u8 *kbase, f32x16 &snext, const f32x16 &s, bf16x8 (&pout)[2],
                    const lds_u8 *vnext, bool do_dma, int dma_tile, bool do_tr, int tr_tile, const lds_u8 *bias_next) {
        bf16x8 kf[KB];
        float m_use = 0.f, psum = 0.f, pe_even = 0.f, pe_prev = 0.f, dnext = 0.f, mxa[5], mx = 0.f, m_new = 0.f;
        u32x4 pw[2];
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 bias_c = zero;
        int e_done = 0;   // softmax elements finished so far (compile-time after unrolling)
        PC_FENCE();
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (i < 2 * DB) {
                o_acc[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], pp[i / DB], o_acc[i % DB], 0, 0, 0);
            } else {
                const int kb = i - 2 * DB;
                snext = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb], qf[0][kb], kb == 0 ? (ALIBI ? bias_c : zero) : snext, 0, 0, 0);
            }
            // ALIBI: the per-key bias of the sub-tile whose scores start at slot 8 enters as the initial
            // accumulator of its K.Q chain, so it costs four LDS reads and no arithmetic
            if constexpr (ALIBI) {
                if (i == 2 * DB - 2) {
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const f32x4 b = *reinterpret_cast<const __attribute__((address_space(3))) f32x4 *>(bias_next + (8 * i4 + 4 * hh) * 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) bias_c[i4 * 4 + e] = b[e];
                    }
                }
            }
            // ---- softmax share of this slot
            if (i == 0) {
#pragma unroll
                for (int c = 0; c < 5; ++c) {
                    mxa[c] = fmaxf(fmaxf(s[3 * c], s[3 * c + 1]), s[3 * c + 2]);
                    asm volatile("" : "+v"(mxa[c]));
                }
            } else if (i == 1) {
                mx = fmaxf(fmaxf(fmaxf(mxa[0], mxa[1]), mxa[2]), fmaxf(fmaxf(mxa[3], mxa[4]), s[15]));
                mx = max_across_halves(mx);
                asm volatile("" : "+v"(mx));
            } else if (i == 2) {
                m_new = mx > m_run + kMaxSlack ? mx : m_run;
                m_use = (m_new == -INFINITY) ? 0.f : m_new;
                asm volatile("" : "+v"(m_use));
            } else if (i == 3) {
                // the reference moves rarely: the rescale factor and the flag that makes rescale() act are set
                // behind a wave-uniform branch
                if (__any(m_new != m_run)) {
                    alpha = __builtin_amdgcn_exp2f(m_run - m_use);
                    rescale_pending = true;
                }
                m_run = m_new;
                dnext = s[0] - m_use;
                asm volatile("" : "+v"(dnext));
            } else {
                const int n_e = i < 8 ? 2 : 1;   // slots 4..7 take two elements, slots 8..15 one
#pragma unroll
                for (int r = 0; r < n_e; ++r) {
                    const int e = e_done + r;
                    // The exp of element e is issued here; its consumers (row sum, bf16 pack) handle
                    // element e-1, whose exp has long finished: nothing waits for a transcendental.
                    float pe = __builtin_amdgcn_exp2f(dnext);
                    asm volatile("" : "+v"(pe));
                    if (e < 15) {
                        dnext = s[e + 1] - m_use;
                        asm volatile("" : "+v"(dnext));
                    }
                    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                    if (e > 0) {
                        psum += pe_prev;
                        asm volatile("" : "+v"(psum));
                        if ((e - 1) & 1) {
                            bf16x2 pr;
                            pr[0] = (__bf16)pe_even;
                            pr[1] = (__bf16)pe_prev;
                            uint32_t w = __builtin_bit_cast(uint32_t, pr);
                            asm volatile("" : "+v"(w));
                            pw[(e - 1) >> 3][((e - 1) & 7) >> 1] = w;
                        } else {
                            pe_even = pe_prev;
                        }
                    }
                    pe_prev = pe;
                    if (e == 15) {   // the last element has no later slot
                        psum += pe;
                        bf16x2 pr;
                        pr[0] = (__bf16)pe_even;
                        pr[1] = (__bf16)pe;
                        pw[1][3] = __builtin_bit_cast(uint32_t, pr);
                    }
                }
                e_done += n_e;
            }
            // ---- operand fragments: slot i < 8 has just used V fragment i, whose registers take K fragment i
            // (used by slot 8+i); slot 8+i has just used K fragment i and reads V fragment i of the next step
            if (i < KB) kf[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const lds_u32x4 *>(kbase + koff(i)));
            else read_v(vnext, i - KB);
            if (do_dma && i < DMA_PER_TILE) whole_piece(dma_tile, i);
            // re-layout of the V tile that became visible at the last barrier
            if (do_tr && i < FRAG_PER_WAVE) transpose_read(tr_tile, i);
            if (do_tr && i >= 4 && i < 4 + FRAG_PER_WAVE) transpose_write(tr_tile, i - 4);
            PC_FENCE();
        }
        l_run = l_run * alpha + psum;
        pout[0] = __builtin_bit_cast(bf16x8, pw[0]);
        pout[1] = __builtin_bit_cast(bf16x8, pw[1]);
        PC_FENCE();
    };
    static_assert(KB == 2 * DB, "slot layout: as many P.V as K.Q matrix instructions per step");

    auto apply_mask = [&](f32x16 &s, int buf, int sub, int n_valid) {
        const lds_u8 *pp = lds + LDS_POS + buf * KT * 4;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const int key0 = sub * 32 + 8 * i4 + 4 * hh;
            const u32x4 kp = *reinterpret_cast<const lds_u32x4 *>(pp + key0 * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((int)kp[e] > qt[0].qpos || key0 + e >= n_valid) s[i4 * 4 + e] = -INFINITY;
        }
    };

    // ALIBI: s += slope * (pos_k - ref) in the log2 domain, ref = the wave's smallest query position.  The
    // term -slope * (pos_q - ref) that completes -slope * (pos_q - pos_k) is the same for every key of a
    // query and cancels in the softmax, so only a per-key value is added.  The difference is taken in
    // integers first: the bias is exact where it is small, i.e. for the keys that carry weight.  The wave
    // computes the 64 values of a tile once, one key per lane (tile_needs_mask has the position in that
    // layout anyway), and passes them to itself through a private strip of LDS to get them into the
    // score layout.
    auto store_bias = [&](int t, int kpos) {
        if constexpr (ALIBI) {
            const float b = slope2 * (float)(kpos - bias_ref);
            *reinterpret_cast<__attribute__((address_space(3))) float *>(lds + LDS_BIAS + (wave * 2 + (t & 1)) * KT * 4 + lane * 4) = b;
        }
    };
    auto bias_strip = [&](int t, int sub) -> const lds_u8 * {
        return lds + LDS_BIAS + (wave * 2 + (t & 1)) * KT * 4 + sub * 32 * 4;
    };
    auto apply_bias = [&](f32x16 &s, int t, int sub) {   // a first sub-tile only: its scores are computed outside a step
        const lds_u8 *bp = lds + LDS_BIAS + (wave * 2 + (t & 1)) * KT * 4;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const int key0 = sub * 32 + 8 * i4 + 4 * hh;
            const f32x4 b = *reinterpret_cast<const __attribute__((address_space(3))) f32x4 *>(bp + key0 * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[i4 * 4 + e] += b[e];
        }
    };

    auto rescale = [&]() {
        if (rescale_pending) {
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) o_acc[b][i] *= alpha;
            alpha = 1.f;
            rescale_pending = false;
        }
    };

    // What does tile t (already visible in LDS) hold for this wave?  A position ID above the wave's smallest
    // query position, or fewer than 64 real keys: the per-element mask is needed.  No position ID at or below
    // the wave's largest query position: nothing to see.  The decision comes in two parts, so that the LDS
    // read's latency can pass behind other work: the position ID of this lane's key of tile t, and the votes.
    auto tile_pos = [&](int t) -> int {
        return *reinterpret_cast<const __attribute__((address_space(3))) int *>(lds + LDS_POS + (t & (NBUF - 1)) * KT * 4 + lane * 4);
    };
    auto tile_vote = [&](int t, int kpos) -> bool {
        const int n_valid = k_end - (k_begin + t * KT);
        store_bias(t, kpos);
        return __any(kpos > wave_min_qpos) || n_valid < KT;
    };
    // (PAGED keeps to the mask: its per-lane addresses leave no registers for the second mode of the loop)
    auto tile_hidden = [&](int kpos) -> bool { return PAGED ? false : !__any(kpos <= wave_max_qpos); };

    // Scores of tile t's first 32 keys into sc[0], and 8 KiB of finite numbers from `stand_in` into vf in place of
    // the V fragments of "the previous sub-tile" (whose P is set to 0): the state in which the loop takes up tile t.
    // K of tile t and the stand-in must be visible.
    auto prime = [&](int t, const lds_u8 *stand_in) {
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const lds_u8 *kbase = lds + LDS_K + (t & (NBUF - 1)) * TILE_BYTES;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const bf16x8 kfr = __builtin_bit_cast(bf16x8, *reinterpret_cast<const lds_u32x4 *>(kbase + koff(kb)));
            sc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, qf[0][kb], kb == 0 ? zero16 : sc[0], 0, 0, 0);
        }
#pragma unroll
        for (int g = 0; g < 2 * DB; ++g) read_v(stand_in, g);
        if constexpr (ALIBI) apply_bias(sc[0], t, 0);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[1][j][e] = (__bf16)0.f;
    };
    // O += V^T.P of the last sub-tile a step has produced P for
    auto drain = [&]() {
        rescale();
#pragma unroll
        for (int i = 0; i < 2 * DB; ++i) o_acc[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], pf[1][i / DB], o_acc[i % DB], 0, 0, 0);
    };

    // ---- main loop
    if (n_tiles > 0) {
        // tile 0 has landed in every wave's eyes after this barrier, and nobody reads staged Q any more
        __syncthreads();
        issue_tile(2);
        bool mask_cur = tile_vote(0, tile_pos(0));
        // V of tile 0 into fragment order; the loop's first barrier publishes it (no barrier of its own)
#pragma unroll
        for (int k = 0; k < FRAG_PER_WAVE; ++k) transpose_read(0, k);
#pragma unroll
        for (int k = 0; k < FRAG_PER_WAVE; ++k) transpose_write(0, k);

        // a wave without a row tile (fewer than 8 row tiles in this block) only helps with staging: its
        // share of the copies and of the V re-layout, and the barriers; the matrix pipe of its SIMD is
        // left to the wave that has work
        const bool idle_wave = rb * kWideRowTilesPerWg + wave * NQT >= row_tiles;
        // Per tile, ONE workgroup barrier at the top.  It makes visible what the iteration reads for the
        // first time: the staged K, V and position IDs of tile t+1 (copies issued two iterations ago) and
        // the V^T fragments of tile t (written during the previous iteration).  Everything an iteration
        // overwrites was last read before that barrier: the copies of tile t+3 go into the K buffer of
        // tile t-1 and the raw-V buffer of tile t, the V^T fragments of tile t+1 replace those of tile t-1.
        for (int t = 0; idle_wave && t < n_tiles; ++t) {
            PC_WAIT_VMCNT(DMA_PER_TILE);
            __syncthreads();
            issue_tile(t + 3);
#pragma unroll
            for (int k = 0; k < FRAG_PER_WAVE; ++k) transpose_read(t + 1, k);
#pragma unroll
            for (int k = 0; k < FRAG_PER_WAVE; ++k) transpose_write(t + 1, k);
        }
        // The wave works on tile t (its first scores are in sc[0]) for as long as tiles hold a key it can see.  When the
        // next tile holds none, it finishes what is in flight and steps aside: for a run of such tiles it only
        // keeps up its share of the staging (and of the barriers) and looks at the following tile's position IDs;
        // it takes up the arithmetic again with the first tile that has a visible key.
        bool live = !idle_wave;
        int t = 0;
        if (live) prime(0, lds + LDS_K);   // the stand-in: tile 0's own keys
        while (live && t < n_tiles) {
            const int buf = t & (NBUF - 1);
            const int n_valid = k_end - (k_begin + t * KT);   // real keys in this tile (may exceed 64)
            const bool has_next = t + 1 < n_tiles;

            // tile t+1 and the V^T fragments of tile t become visible; the copies of tile t+2 may stay in flight.
            // What the barrier publishes of this wave's LDS traffic are its re-laid-out V fragments, written eight
            // or more LDS instructions ago (LDS instructions complete in order): the V fragment reads issued since
            // (the last eight, by the previous step or by prime()) need not have returned.  They read a buffer that
            // is next written a whole step after this barrier.
            // (PAGED looks its row ranges up with scalar loads, which share that counter and return out of
            // order: it waits for everything.)
            if constexpr (PAGED) {
                PC_WAIT_VMCNT(DMA_PER_TILE);
                __syncthreads();
            } else {
                PC_WAIT_VM_LGKM(DMA_PER_TILE, 2 * DB);
                __builtin_amdgcn_s_barrier();
            }
            // tile t+1's position IDs are read now and voted on after the first step (the read returns behind it)
            int kpos_next = tile_pos(has_next ? t + 1 : t);

            const lds_u8 *k_cur = lds + LDS_K + buf * TILE_BYTES;
            const lds_u8 *v_cur = lds + LDS_VT + (t & (NVT - 1)) * TILE_BYTES;   // fragments 0..7: first 32 keys, 8..15: last 32
            // K.Q of the next tile's first half (past the last tile: recomputed on this tile, result unused)
            const lds_u8 *k_nxt = lds + LDS_K + (has_next ? (t + 1) & (NBUF - 1) : buf) * TILE_BYTES;
            if (mask_cur) apply_mask(sc[0], buf, 0, n_valid);
            rescale();
            // P.V of tile t-1's second half | K.Q of this tile's second half | softmax of its first half;
            // the copies of tile t+3 are issued here (inside the step when the tile is whole)
            const bool whole3 = begin_tile(t + 3);
            if (!whole3) ragged_tile(t + 3);
            step(pf[1], k_cur + 32 * ROW_BYTES, sc[1], sc[0], pf[0], v_cur, whole3, t + 3, false, 0, bias_strip(t, 1));
            asm volatile("" : "+v"(kpos_next));
            const bool mask_next = has_next ? tile_vote(t + 1, kpos_next) : false;
            const bool hidden_next = has_next ? tile_hidden(kpos_next) : false;

            if (mask_cur) apply_mask(sc[1], buf, 1, n_valid);
            rescale();
            // P.V of this tile's first half | K.Q of tile t+1's first half | softmax of this tile's second half;
            // V of tile t+1 is brought into fragment order
            step(pf[0], k_nxt, sc[0], sc[1], pf[1], v_cur + 8 * 1024, false, 0, true, t + 1, bias_strip(has_next ? t + 1 : t, 0));
            mask_cur = mask_next;
            ++t;
            if (hidden_next) {   // wave-uniform (and rare)
                drain();
                live = false;
                for (; t < n_tiles; ++t) {   // tile t is hidden
                    const bool more = t + 1 < n_tiles;
                    PC_WAIT_VMCNT(DMA_PER_TILE);
                    __syncthreads();
                    const int kp = tile_pos(more ? t + 1 : t);
                    issue_tile(t + 3);
#pragma unroll
                    for (int k = 0; k < FRAG_PER_WAVE; ++k) transpose_read(t + 1, k);
#pragma unroll
                    for (int k = 0; k < FRAG_PER_WAVE; ++k) transpose_write(t + 1, k);
                    if (more && !tile_hidden(kp)) {
                        mask_cur = tile_vote(t + 1, kp);
                        prime(t + 1, lds + LDS_VT + (t & (NVT - 1)) * TILE_BYTES);   // K of tile t+1 and the V^T fragments of tile t became visible at this barrier
                        live = true;
                        ++t;
                        break;
                    }
                }
            }
        }
        // P.V of the very last sub-tile
        if (live) drain();
    }
    PC_WAIT_VMCNT(0);   // copies past the split's end may still be landing in LDS

    // ---- epilogue: O^T from the accumulators straight to global memory, no LDS and no barrier (a wave is done when
    // its own stores are out).  A lane holds, per 32-row block b of O^T, four groups of 4 consecutive d of its query
    // (d = 32 b + 8 i4 + 4 hh ..).  The two lanes of a query (lane, lane^32) exchange halves, after which lane hh owns
    // the 16 consecutive d = 32 b + 16 hh .. of the query's row: two 16-byte stores per b.  One pass over the keys:
    // the normalised output row; split over the keys: this split's un-normalised O, rounded to bf16, and (m, l),
    // which attn_combine_kernel merges.
    const int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const int col_e = lane_e & 31, hh_e = lane_e >> 5;
    const int rt_e = rb * kWideRowTilesPerWg + wave;
    if (rt_e >= row_tiles) return;   // wave-uniform: a wave without a row tile
    const float l_tot = sum_across_halves(l_run);
    const float scale = a_n_splits == 1 ? (l_tot > 0.f ? 1.f / l_tot : 0.f) : 1.f;
    int g_head_e, tq_e;
    split_row_tile(rt_e, tiles_q, a_G, g_head_e, tq_e);
    const int head = kvh * a_G + g_head_e;
    const int qi_e = tq_e * RW + col_e;
    // the output is [total_q][Hq] rows; a split's partials are [Hq][total_q] rows, so that the 32 rows of a wave are
    // 8 KiB in one piece (rows 8 KiB apart all fall on one memory channel)
    const size_t q_row = (size_t)(seq.q_begin + (qi_e < seq.n_q ? qi_e : 0));
    const size_t out_row = a_n_splits > 1 ? ((size_t)split * a_Hq + head) * p.total_q + q_row : q_row * a_Hq + head;
    uint16_t *dst = (a_n_splits > 1 ? p.part_o : p.out) + out_row * D + hh_e * 16;
#pragma unroll
    for (int b = 0; b < DB; ++b) {
        uint32_t w[4][2];   // [i4][pair of d]
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                bf16x2 pr;
                pr[0] = (__bf16)(o_acc[b][i4 * 4 + 2 * h] * scale);
                pr[1] = (__bf16)(o_acc[b][i4 * 4 + 2 * h + 1] * scale);
                w[i4][h] = __builtin_bit_cast(uint32_t, pr);
            }
        // after the exchange the lower half-wave holds groups 0 and 1 of both lanes of the query, the upper one 2 and 3
        u32x4 c[2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const u32x2 r = __builtin_amdgcn_permlane32_swap(w[j][h], w[j + 2][h], false, false);
                c[j][h] = r[0];       // d + 0..3 of the group (from the lane with hh = 0)
                c[j][2 + h] = r[1];   // d + 4..7 (from the lane with hh = 1)
            }
        if (qi_e < seq.n_q) {
            *reinterpret_cast<u32x4 *>(dst + b * 32) = c[0];
            *reinterpret_cast<u32x4 *>(dst + b * 32 + 8) = c[1];
        }
    }
    if (a_n_splits > 1 && hh_e == 0 && qi_e < seq.n_q) p.part_ml[out_row] = make_float2(m_run, l_tot);
}

template <int NQT, int NW, bool PAGED, bool ALIBI, typename Tab>
int launch_one(pc_ctx *ctx, AttnParams &p, int n_blocks, hipStream_t stream, const Tab &tab)
{
    static bool attr_set[16] = {false};
    auto kern = attn_bf16_dma_kernel<NQT, NW, PAGED, ALIBI>;
    if (!attr_set[ctx->device & 15]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                LDS_TOTAL) != hipSuccess)
            return PC_E_HIP;
        attr_set[ctx->device & 15] = true;
    }
    // the 14 dwords the kernel gets in registers: small integers packed, the first prompt, three pointers
    if (p.Hkv > 255 || p.G > 255 || p.n_splits > 255 || p.n_seqs > 255 || p.Hq >= (1 << 23)) return PC_E_UNSUPPORTED;
    const uint64_t pk = reinterpret_cast<uint64_t>(p.k), pv = reinterpret_cast<uint64_t>(p.v), pp = reinterpret_cast<uint64_t>(p.kv_pos);
    int hkv_shift = 0;
    while ((1 << hkv_shift) < p.Hkv) ++hkv_shift;
    const int share0 = (((p.seq0.n_kv + p.n_splits - 1) / p.n_splits) + KT - 1) & ~(KT - 1);   // keys per split, whole 64-key tiles
    const i32x4 h0 = {hkv_shift, share0, p.Hkv | (p.n_splits << 8) | (p.G << 16) | ((p.q_rotated ? 1 : 0) << 24), p.n_seqs | (int)((unsigned)p.Hq << 8)};
    const i32x4 h1 = {p.seq0.q_begin, p.seq0.n_q, p.seq0.kv_begin, p.seq0.n_kv};
    const i32x4 h2 = {(int)(uint32_t)pk, (int)(uint32_t)(pk >> 32), (int)(uint32_t)pv, (int)(uint32_t)(pv >> 32)};
    const i32x2 h3 = {(int)(uint32_t)pp, (int)(uint32_t)(pp >> 32)};
    (void)n_blocks;
    const dim3 grid((unsigned)(p.rb_max << hkv_shift), (unsigned)p.n_splits, (unsigned)p.n_seqs);
    return launch_kernel(ctx, kProfAttn, kern, grid, dim3(NW * 64), LDS_TOTAL, stream, h0, h1, h2, h3, p, tab);
}

}  // namespace

int launch_attn_bf16_wide(pc_ctx *ctx, attn::AttnParams &p, int n_blocks, hipStream_t stream, const KvSegTable *tab)
{
    if (p.alibi) {
        if (tab) return launch_one<1, 8, true, true>(ctx, p, n_blocks, stream, *tab);
        return launch_one<1, 8, false, true>(ctx, p, n_blocks, stream, NoSegTable{0});
    }
    if (tab) return launch_one<1, 8, true, false>(ctx, p, n_blocks, stream, *tab);
    return launch_one<1, 8, false, false>(ctx, p, n_blocks, stream, NoSegTable{0});
}

}  // namespace pc
