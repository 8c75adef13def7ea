// A prompt's KV as a list of row ranges read in place (Sec. 3.4 of the paper: prompts of a batch share a
// module instead of copying it).  Each range is a module's block in the pool, or the uncached tokens' own
// rows in the caller's tail buffer; the ranges of a prompt follow each other in the prompt's row order.
#pragma once

#include "common.h"

namespace pc {

// Rows of segment s are the prompt's rows [first_row, first_row of s+1); all three pointers address the
// segment's row 0.
struct KvSeg {
    const uint8_t *k;
    const uint8_t *v;
    const int32_t *pos;
    int first_row;
    int pad_;
};
constexpr int kMaxKvSegs = 64;
struct KvSegTable {
    int seg_begin[kMaxAttnSeqs + 1];   // prompt i owns seg[seg_begin[i] .. seg_begin[i+1])
    KvSeg seg[kMaxKvSegs];
};

// Walks one prompt's ranges in increasing row order.  The table lives in the kernel arguments and is only
// indexed with wave-uniform values; the range that holds the row of the last advance_to() is kept in
// registers, so rows of that range cost one multiply-add, and only rows beyond it look further.
struct KvSegWalker {
    const KvSegTable *tab;
    int lo, n, cur;
    uint32_t cur_first, next_first;
    const uint8_t *k, *v;
    const int32_t *pos;

    __device__ __forceinline__ void load(int e)
    {
        const KvSeg sg = tab->seg[__builtin_amdgcn_readfirstlane(lo + e)];
        k = sg.k;
        v = sg.v;
        pos = sg.pos;
        cur_first = (uint32_t)sg.first_row;
        next_first = e + 1 < n ? (uint32_t)tab->seg[__builtin_amdgcn_readfirstlane(lo + e + 1)].first_row : 0xffffffffu;
    }
    __device__ __forceinline__ void init(const KvSegTable *t, int seq_i)
    {
        tab = t;
        lo = t->seg_begin[seq_i];
        n = t->seg_begin[seq_i + 1] - lo;
        cur = 0;
        load(0);   // a prompt with query rows has at least the range of its own tokens
    }
    // row (wave-uniform, not below the row of an earlier call): first row the coming lookups can touch
    __device__ __forceinline__ void advance_to(uint32_t row)
    {
        while (next_first <= row) load(++cur);
    }
    // row (per lane, >= the row of the last advance_to, < row_hi with row_hi wave-uniform): addresses of that
    // row's K and V (byte offset head_off inside a row of row_bytes bytes) and of its position ID
    __device__ __forceinline__ void locate(uint32_t row, uint32_t row_hi, uint32_t row_bytes, uint32_t head_off,
                                           const uint8_t *&kp, const uint8_t *&vp, const int32_t *&pp) const
    {
        const uint8_t *bk = k, *bv = v;
        const int32_t *bp = pos;
        uint32_t first = cur_first;
        if (next_first < row_hi) {   // the rows asked for run into later ranges
            for (int sx = cur + 1; sx < n; ++sx) {
                const KvSeg sg = tab->seg[__builtin_amdgcn_readfirstlane(lo + sx)];
                if ((uint32_t)sg.first_row >= row_hi) break;
                const bool in = row >= (uint32_t)sg.first_row;
                bk = in ? sg.k : bk;
                bv = in ? sg.v : bv;
                bp = in ? sg.pos : bp;
                first = in ? (uint32_t)sg.first_row : first;
            }
        }
        const uint32_t local = row - first;
        const size_t off = (size_t)local * row_bytes + head_off;
        kp = bk + off;
        vp = bv + off;
        pp = bp + local;
    }
};

}  // namespace pc
