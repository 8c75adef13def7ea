// Internal declarations shared by the host runtime and the kernel launchers.
// Nothing here is part of the public ABI (see include/promptcache.h).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include <unordered_map>
#include <vector>

#include "promptcache.h"

namespace pc {

// One stored prompt module of one layer: where its K block starts in the pool
// (the V block follows it), how many rows it has and its first position ID.
struct ModuleEntry {
    size_t k_offset;
    size_t v_offset;
    int n_tokens;
    int start_pos;
    bool host = false;   // offsets are into the pinned host pool (Sec. 4.1, modules kept in CPU memory)
};

// A scaffold (Sec. 3.3): modules that were also encoded jointly; override[i] names the stored states that
// replace member[i] when a prompt imports every member.
struct Scaffold {
    std::vector<int> member, override_id;
};

// Heap allocations made by the request path's planning code are counted (pc_plan_stats), so that a test can show
// that a call whose plan is cached makes none.
extern thread_local long g_plan_heap_allocs;
template <typename T>
struct CountingAlloc {
    using value_type = T;
    CountingAlloc() = default;
    template <typename U>
    CountingAlloc(const CountingAlloc<U> &) {}
    T *allocate(size_t n)
    {
        ++g_plan_heap_allocs;
        return static_cast<T *>(::operator new(n * sizeof(T)));
    }
    void deallocate(T *p, size_t) { ::operator delete(p); }
    template <typename U>
    bool operator==(const CountingAlloc<U> &) const { return true; }
    template <typename U>
    bool operator!=(const CountingAlloc<U> &) const { return false; }
};
template <typename T>
using cvec = std::vector<T, CountingAlloc<T>>;

// The validated import lists of one call (Sec. 3.4: a prompt's imports are checked against the schema and its
// modules retrieved once per prompt, not once per layer).  Everything in it is independent of the layer:
// which stored states each prompt concatenates, in which order, how many rows, at which position IDs.
// Per layer only the modules' addresses differ; they are looked up for every layer when the plan is made.
struct PlanItem {
    int prompt;      // index of the prompt in the call
    int module_id;   // after scaffold overrides
    int n_rows;      // > 0 (modules without tokens are dropped)
    int start_pos;
    int row;         // first row inside the prompt's span
};
struct Plan {
    // key
    cvec<int> ids, mod_offsets;
    unsigned long generation = 0;   // of the context's module tables and scaffolds when the plan was made
    // value
    cvec<PlanItem> items;
    cvec<int> prompt_rows;                      // module rows per prompt
    cvec<const ModuleEntry *> entry;            // [layer][item]
    cvec<unsigned char> layer_ok;               // the layer holds every item with the plan's length and first position
    unsigned long last_use = 0;
    bool valid = false;
};
constexpr int kPlanCacheSize = 8;

// A parameter of a module (Sec. 3.2.2): rows [offset, offset+len) of the module hold placeholder states.
struct ParamSlot {
    int offset;
    int len;
};

// Optional per-kernel timing with HIP events recorded on the caller's stream right
// around each kernel launch (off by default; see pc_profile_enable).
enum ProfKind { kProfGather = 0, kProfAppend = 1, kProfAttn = 2, kProfCombine = 3, kProfRope = 4, kProfKinds = 5 };
struct Profiler {
    int capacity = 0;  // event pairs per kind; 0 = disabled
    std::vector<hipEvent_t> start[kProfKinds], stop[kProfKinds];
    int used[kProfKinds] = {0, 0, 0, 0, 0};
};

// How the last attention call was decomposed (reported to benchmarks).
struct AttnLaunchInfo {
    int n_splits = 0;
    int n_workgroups = 0;
    int waves_per_wg = 0;
};

}  // namespace pc

struct pc_ctx {
    pc_config cfg;
    int device = 0;
    int elem_bytes = 0;
    size_t row_bytes = 0;  // n_kv_heads * head_dim * elem_bytes

    uint8_t *pool = nullptr;  // module pool (device)
    size_t pool_used = 0;
    uint8_t *host_pool = nullptr;  // module pool in pinned host memory, mapped into the device's address space
    size_t host_pool_bytes = 0, host_pool_used = 0;
    int host_copy_mode = PC_HOST_READ_KERNEL;
    int attn_kernel = PC_ATTN_AUTO;
    std::vector<std::unordered_map<int, pc::ModuleEntry>> modules;  // per layer
    std::unordered_map<int, std::vector<pc::ParamSlot>> params;     // per module id (schema level, all layers)
    std::vector<pc::Scaffold> scaffolds;                            // in definition order (schema level)
    unsigned long generation = 1;   // bumped by every change of the tables above that can change a plan
    pc::Plan plans[pc::kPlanCacheSize];
    unsigned long plan_clock = 0, plan_hits = 0, plan_misses = 0;

    float2 *rope_table = nullptr;  // device, [max_pos][head_dim/2] (cos, sin)
    int32_t *iota = nullptr;  // device, 0, 1, .. max_pos-1: position IDs of module rows read in place
    float2 *rope_table_t = nullptr;  // the same values as [head_dim/2][max_pos]: coalesced when lanes hold consecutive positions

    float *alibi = nullptr;    // device [n_q_heads] slopes of the linear bias (Sec. 4.2); allocated always
    bool use_alibi = false;    // position encoding in force: false = rotation (RoPE), true = linear bias (ALiBi)

    float *scratch = nullptr;  // device, split-KV partials
    size_t scratch_bytes = 0;
    uint8_t *static_scratch = nullptr;  // this device's copy of the library's fixed scratch array (pc_prefill_attn_static)

    int n_cu = 256;
    pc::AttnLaunchInfo last_attn;
    pc::Profiler prof;
};

namespace pc {

// ---- gather (KV assembly) ---------------------------------------------------
// One contiguous run of rows copied from the pool to the packed output.
struct GatherSeg {
    const uint8_t *src_k;   // nullptr: the rows are brought in by a copy-engine transfer, the kernel writes
    const uint8_t *src_v;   //          their position IDs only (tiles of kPosOnlyTileFactor x rows_per_tile rows)
    int dst_row;     // first output row
    int n_rows;
    int start_pos;   // position ID of the first row
    int first_tile;  // index of this segment's first tile in the launch
};

constexpr int kMaxGatherSegs = 64;
constexpr int kPosOnlyTileFactor = 64;

struct GatherArgs {
    int n_segs;
    int total_tiles;
    int rows_per_tile;
    int row_bytes;
    GatherSeg seg[kMaxGatherSegs];
};

int launch_gather(pc_ctx *ctx, const GatherArgs &args, uint8_t *out_k, uint8_t *out_v, int32_t *out_pos,
                  hipStream_t stream);

// The imported modules of several layers in one launch: every segment names the layer whose packed buffers it
// is copied into (the modules do not depend on the forward pass, Sec. 3.4, so all layers' copies can be made at
// the start of a request).
constexpr int kMaxGatherLayers = 32;
struct GatherLayerOut {
    uint8_t *k, *v;
    int32_t *pos;
};
struct GatherLayersArgs {
    GatherArgs g;
    unsigned char seg_layer[kMaxGatherSegs];   // index into out[]
    GatherLayerOut out[kMaxGatherLayers];
};
int launch_gather_layers(pc_ctx *ctx, const GatherLayersArgs &args, hipStream_t stream);

// ---- RoPE / append -----------------------------------------------------------
int launch_rope(pc_ctx *ctx, void *x, int n_tokens, int n_heads, const int32_t *pos, hipStream_t stream);

// One prompt's slice for the batched append: rows [q_begin, q_begin+n) of the new
// tokens go to rows [dst_row, dst_row+n) of the packed KV.
struct AppendSeg {
    int q_begin;
    int n;
    int dst_row;
    int pos0;   // kPosFromArray: position IDs come from the q_pos array; kPosMaskRows: the rows only lose
                // their position (no token there any more); >= 0: row r gets position pos0 + r
};
constexpr int kPosFromArray = -1;
constexpr int kPosMaskRows = -2;
constexpr int kMaxAppendSegs = 128;
struct AppendArgs {
    int n_segs;
    int total_rows;
    AppendSeg seg[kMaxAppendSegs];
};
// Assembly and append of a batch in one launch (at most kMaxFusedAppendSegs prompts).
constexpr int kMaxFusedAppendSegs = 64;
struct FusedKvArgs {
    GatherArgs g;
    int n_app;
    int app_rows;
    AppendSeg app[kMaxFusedAppendSegs];
};
// q_new != nullptr: the launch also writes q_rot[row] = rotation of q_new[row] at the row's position, times q_scale
int launch_gather_append(pc_ctx *ctx, const FusedKvArgs &args, uint8_t *out_k, uint8_t *out_v, int32_t *out_pos,
                         const void *k_new, const void *v_new, const int32_t *q_pos, hipStream_t stream,
                         const void *q_new = nullptr, void *q_rot = nullptr, float q_scale = 1.f);

int launch_append(pc_ctx *ctx, const AppendArgs &args, const void *k_new, const void *v_new, const int32_t *q_pos,
                  void *asm_k, void *asm_v, int32_t *asm_pos, hipStream_t stream, const void *q_new = nullptr,
                  void *q_rot = nullptr, float q_scale = 1.f);

// ---- attention -----------------------------------------------------------------
// One prompt of a (possibly batched) attention call.
struct AttnSeq {
    int q_begin;   // first query row in Q_new / out
    int n_q;
    int kv_begin;  // first row in the packed KV
    int n_kv;
};
constexpr int kMaxAttnSeqs = 64;
struct AttnBatch {
    int n_seqs;
    AttnSeq seq[kMaxAttnSeqs];
};

// Where an attention launch keeps its split-KV partials.  strict: a launch whose partials do not fit is refused
// (PC_E_CAPACITY) instead of being run with fewer splits.
struct ScratchRef {
    uint8_t *ptr;
    size_t bytes;
    bool strict;
};

struct KvSegTable;
int launch_attn_f32(pc_ctx *ctx, const AttnBatch &batch, const float *q, const int32_t *q_pos, const float *k,
                    const float *v, const int32_t *kv_pos, float *out, hipStream_t stream, const KvSegTable *tab = nullptr,
                    bool q_rotated = false);

int launch_attn_bf16(pc_ctx *ctx, const AttnBatch &batch, const void *q, const int32_t *q_pos, const void *k,
                     const void *v, const int32_t *kv_pos, void *out, hipStream_t stream, const KvSegTable *tab = nullptr,
                     bool q_rotated = false, const ScratchRef *scratch = nullptr /* nullptr: the context's own */);

inline int hip_status(hipError_t e) { return e == hipSuccess ? PC_OK : PC_E_HIP; }

// Launch a kernel on `stream`.  When profiling is on and an event pair of `kind` is free, the
// launch carries the pair (hipExtLaunchKernelGGL), so the pair reads the kernel's own begin and
// end timestamps rather than the time between two stream markers.
template <typename... Args, typename F = void (*)(Args...)>
inline int launch_kernel(pc_ctx *ctx, int kind, F kernel, dim3 grid, dim3 block, unsigned smem, hipStream_t stream,
                         Args... args)
{
    Profiler &p = ctx->prof;
    if (p.capacity > 0 && p.used[kind] < p.capacity) {
        const int slot = p.used[kind]++;
        hipExtLaunchKernelGGL(kernel, grid, block, smem, stream, p.start[kind][slot], p.stop[kind][slot], 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, smem, stream, args...);
    }
    return hip_status(hipGetLastError());
}

}  // namespace pc
