// Host runtime of the Prompt Cache hot path: context, module pool, request planning
// (which pool rows go where, validation of the imported modules) and the C ABI.
// All numerical work happens in the kernels; this file only moves integers and
// pointers.  See include/promptcache.h for the contract of every entry point.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <new>

#include "common.h"
#include "attn_bf16.h"

using namespace pc;

thread_local long pc::g_plan_heap_allocs = 0;

static __device__ __align__(256) uint8_t scratch[PC_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t kPoolAlign = 256;
constexpr size_t kDefaultScratch = (size_t)256 << 20;

// Fixed scratch of pc_prefill_attn_static: split-KV partials of callers that must not allocate.  Every GPU the
// library runs on holds its own copy of the array (until the process ends) at its own address; in host code the
// array's name is only a handle for hipGetSymbolAddress, never a device address.  pc_create looks the address up
// once per device and every later use goes through that pointer.
constexpr size_t kStaticScratchBytes = (size_t)PC_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
uint8_t *g_static_scratch[kMaxDevices] = {nullptr};   // per device, filled by pc_create with that device current

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

int elem_size(int dtype) { return dtype == PC_F32 ? 4 : (dtype == PC_BF16 ? 2 : 0); }

int validate_config(const pc_config *c)
{
    if (!c) return PC_E_BADARG;
    if (c->n_layers <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0) return PC_E_BADARG;
    if (c->n_q_heads % c->n_kv_heads) return PC_E_BADARG;
    if (c->max_pos <= 0 || !(c->rope_base > 1.0)) return PC_E_BADARG;
    if (c->dtype == PC_BF16) {
        if (c->head_dim != 64 && c->head_dim != 128) return PC_E_UNSUPPORTED;
    } else if (c->dtype == PC_F32) {
        if ((c->head_dim & 3) || c->head_dim > 256) return PC_E_UNSUPPORTED;  // rows must be 16-byte multiples
    } else {
        return PC_E_UNSUPPORTED;
    }
    return PC_OK;
}

// Sorted-interval test: do any two [start, start+len) ranges share a position ID?
int check_ranges(int n, const int *starts, const int *lens, int max_pos)
{
    if (n < 0 || (n > 0 && (!starts || !lens))) return PC_E_BADARG;
    cvec<std::pair<long, long>> iv;
    iv.reserve(n);
    for (int i = 0; i < n; ++i) {
        if (lens[i] < 0 || starts[i] < 0) return PC_E_BADARG;
        if ((long)starts[i] + lens[i] > (long)max_pos) return PC_E_POS_RANGE;
        if (lens[i] > 0) iv.emplace_back(starts[i], (long)starts[i] + lens[i]);
    }
    std::sort(iv.begin(), iv.end());
    for (size_t i = 1; i < iv.size(); ++i)
        if (iv[i].first < iv[i - 1].second) return PC_E_OVERLAP;
    return PC_OK;
}

// Scaffolding (Sec. 3.3): replace, in place, the ids of every scaffold whose members are all in the list by
// the ids of its jointly encoded states.  Scaffolds are taken in definition order; one that would touch a
// member an earlier scaffold has overridden is skipped.
void apply_scaffolds(const std::vector<Scaffold> &scaffolds, cvec<int> &ids, cvec<int> *replaced_from = nullptr)
{
    if (replaced_from) *replaced_from = ids;
    if (scaffolds.empty() || ids.empty()) return;
    const cvec<int> imported(ids);
    cvec<int> taken;
    auto has = [](const cvec<int> &v, int x) { return std::find(v.begin(), v.end(), x) != v.end(); };
    for (const Scaffold &sc : scaffolds) {
        bool complete = true;
        for (int m : sc.member) complete = complete && has(imported, m) && !has(taken, m);
        if (!complete) continue;
        for (size_t i = 0; i < sc.member.size(); ++i) {
            for (size_t j = 0; j < ids.size(); ++j)
                if (imported[j] == sc.member[i] && !has(taken, imported[j])) ids[j] = sc.override_id[i];
            taken.push_back(sc.member[i]);
        }
    }
}

// ---- request planning (Sec. 3.4: the imports of a prompt are validated and its modules retrieved once) --------
//
// make_plan does the whole validation of a call's import lists against the module table of one layer: scaffold
// overrides, look-up of every id, position ranges of a prompt's modules disjoint, rows fit the prompt's span.
// Its result does not depend on the layer as long as the layer stores the same modules with the same lengths
// and first position IDs, which mark_layers establishes for every layer at once.  get_plan keeps the last few
// plans: a call with the import lists of an earlier one (the next layer of the same prompt, the next step of a
// serving loop) compares integers and allocates nothing.

const ModuleEntry *find_module(const pc_ctx *ctx, int layer, int id)
{
    const auto &table = ctx->modules[layer];
    auto it = table.find(id);
    return it == table.end() ? nullptr : &it->second;
}

// Rows available to prompt b: kv_offsets[b+1] - kv_offsets[b], of which its q_offsets[b+1] - q_offsets[b] uncached
// tokens need their share (q_offsets == nullptr: none; kv_offsets == nullptr: capacity not checked here).
long rows_available(const int *kv_offsets, const int *q_offsets, int b)
{
    return (long)kv_offsets[b + 1] - kv_offsets[b] - (q_offsets ? (long)q_offsets[b + 1] - q_offsets[b] : 0L);
}

int make_plan(const pc_ctx *ctx, int layer, const int *ids_flat, const int *mod_offsets, int n_prompts,
              const int *kv_offsets, const int *q_offsets, Plan &p, cvec<int> &member_of)
{
    p.valid = false;
    p.items.clear();
    p.prompt_rows.assign(n_prompts, 0);
    member_of.clear();
    cvec<int> resolved, from, starts, lens;
    for (int b = 0; b < n_prompts; ++b) {
        const int n = mod_offsets[b + 1] - mod_offsets[b];
        const int *ids = n > 0 ? ids_flat + mod_offsets[b] : nullptr;
        resolved.assign(ids, ids + n);
        apply_scaffolds(ctx->scaffolds, resolved, &from);
        for (int i = 0; i < n; ++i) {   // an override must mirror its member (same length, same first position ID)
            if (resolved[i] == from[i]) continue;
            const ModuleEntry *o = find_module(ctx, layer, resolved[i]);
            if (!o) return PC_E_UNKNOWN_MODULE;
            const ModuleEntry *m = find_module(ctx, layer, from[i]);
            if (m && (m->n_tokens != o->n_tokens || m->start_pos != o->start_pos)) return PC_E_SCHEMA;
        }
        starts.resize(n);
        lens.resize(n);
        long rows = 0;
        for (int i = 0; i < n; ++i) {
            const ModuleEntry *m = find_module(ctx, layer, resolved[i]);
            if (!m) return PC_E_UNKNOWN_MODULE;
            starts[i] = m->start_pos;
            lens[i] = m->n_tokens;
            rows += lens[i];
        }
        int rc = check_ranges(n, starts.data(), lens.data(), ctx->cfg.max_pos);
        if (rc != PC_OK) return rc;
        if (rows > 0x7fffffffL || (kv_offsets && rows > rows_available(kv_offsets, q_offsets, b))) return PC_E_CAPACITY;
        int row = 0;
        for (int i = 0; i < n; ++i) {
            p.items.push_back(PlanItem{b, resolved[i], lens[i], starts[i], row});
            member_of.push_back(from[i]);
            row += lens[i];
        }
        p.prompt_rows[b] = (int)rows;
    }
    return PC_OK;
}

// For every layer: the addresses of the plan's modules there, and whether the layer agrees with the plan
// (every module stored, same length and first position ID, overrides mirroring their members).
void mark_layers(const pc_ctx *ctx, Plan &p, const cvec<int> &member_of)
{
    const int L = ctx->cfg.n_layers;
    const size_t n = p.items.size();
    p.entry.assign((size_t)L * n, nullptr);
    p.layer_ok.assign(L, 1);
    for (int layer = 0; layer < L; ++layer)
        for (size_t i = 0; i < n; ++i) {
            const PlanItem &it = p.items[i];
            const ModuleEntry *m = find_module(ctx, layer, it.module_id);
            bool ok = m && m->n_tokens == it.n_rows && m->start_pos == it.start_pos;
            if (ok && member_of[i] != it.module_id) {
                const ModuleEntry *mem = find_module(ctx, layer, member_of[i]);
                ok = !mem || (mem->n_tokens == it.n_rows && mem->start_pos == it.start_pos);
            }
            p.entry[(size_t)layer * n + i] = m;
            if (!ok) p.layer_ok[layer] = 0;
        }
}

struct PlanRef {
    const Plan *plan = nullptr;
    const ModuleEntry *const *entry = nullptr;   // this layer's modules, one per plan item
};

// The plan for these import lists at this layer: from the cache, or made now (and cached).  Errors are those of
// make_plan.
int get_plan(pc_ctx *ctx, int layer, const int *ids_flat, const int *mod_offsets, int n_prompts, const int *kv_offsets,
             const int *q_offsets, PlanRef &out)
{
    const int n_ids = mod_offsets[n_prompts] - mod_offsets[0];
    for (int b = 0; b < n_prompts; ++b)
        if (mod_offsets[b + 1] < mod_offsets[b]) return PC_E_BADARG;
    if (n_ids > 0 && !ids_flat) return PC_E_BADARG;
    Plan *hit = nullptr;
    for (Plan &p : ctx->plans) {
        if (!p.valid || p.generation != ctx->generation || (int)p.mod_offsets.size() != n_prompts + 1 ||
            (int)p.ids.size() != n_ids || !p.layer_ok[layer])
            continue;
        bool same = true;
        for (int b = 0; b <= n_prompts && same; ++b) same = p.mod_offsets[b] == mod_offsets[b] - mod_offsets[0];
        if (same && (n_ids == 0 || memcmp(p.ids.data(), ids_flat + mod_offsets[0], (size_t)n_ids * sizeof(int)) == 0)) {
            hit = &p;
            break;
        }
    }
    if (hit) {
        if (kv_offsets)
            for (int b = 0; b < n_prompts; ++b)
                if (hit->prompt_rows[b] > rows_available(kv_offsets, q_offsets, b)) return PC_E_CAPACITY;
        ++ctx->plan_hits;
    } else {
        ++ctx->plan_misses;
        Plan *victim = &ctx->plans[0];
        for (Plan &p : ctx->plans) {
            if (!p.valid) { victim = &p; break; }
            if (p.last_use < victim->last_use) victim = &p;
        }
        cvec<int> member_of;
        int rc = make_plan(ctx, layer, ids_flat, mod_offsets, n_prompts, kv_offsets, q_offsets, *victim, member_of);
        if (rc != PC_OK) return rc;
        victim->ids.assign(ids_flat + (n_ids ? mod_offsets[0] : 0), ids_flat + (n_ids ? mod_offsets[0] : 0) + n_ids);
        victim->mod_offsets.resize(n_prompts + 1);
        for (int b = 0; b <= n_prompts; ++b) victim->mod_offsets[b] = mod_offsets[b] - mod_offsets[0];
        victim->generation = ctx->generation;
        mark_layers(ctx, *victim, member_of);
        victim->valid = true;
        hit = victim;
    }
    hit->last_use = ++ctx->plan_clock;
    out.plan = hit;
    out.entry = hit->entry.data() + (size_t)layer * hit->items.size();
    return PC_OK;
}

// A host-resident module under PC_HOST_COPY_ENGINE is brought in by copy-engine transfers; the kernel then
// writes its rows' position IDs only.
bool by_copy_engine(const pc_ctx *ctx, const ModuleEntry *m) { return m->host && ctx->host_copy_mode == PC_HOST_COPY_ENGINE; }

// Rows per tile of a gather launch.  All workgroups of a launch are resident at once and the launch lasts as long as
// its busiest CU, so the tile size is the one that gives the busiest CU the fewest bytes when workgroup i runs on CU
// i mod n_cu: tiles first, then `extra_wgs` workgroups that move `extra_bytes` each (the appended rows of the fused
// launch).  Candidates are 32, 24 and 16 KiB of K (and as much of V) per tile; ties go to the larger tile.  (Measured,
// one module of 2 KiB rows: 512 tiles of 32 KiB 11.7 us, 528 tiles 15.1 us, the same 8448 rows in 704 tiles of 24 KiB
// 12.6 us; rows of 8 KiB, 2112 rows and 128 appended rows: 528 tiles 15.5 us, 705 tiles of 24 KiB 12.8 us.)
// A workgroup moves a tile in one pass (512 lanes x 4 x 16 bytes of K and of V, all loads issued before the first
// store).  Launches of more than 128 MiB take 64 KiB tiles, two passes per workgroup (~6 % faster there).
// `n_layers` layers' modules go into the launch.
int gather_rows_per_tile(const pc_ctx *ctx, const PlanRef &pr, long extra_wgs = 0, int n_layers = 1, size_t extra_bytes = 0)
{
    const size_t n = pr.plan->items.size();
    size_t rows = 0;
    for (const PlanItem &it : pr.plan->items) rows += (size_t)it.n_rows;
    const size_t rb = ctx->row_bytes;
    if (rows * n_layers * rb > ((size_t)128 << 20)) return std::max(1, (int)(65536 / rb));
    const long n_cu = ctx->n_cu > 0 ? ctx->n_cu : 256;
    auto tiles_with = [&](int rpt) {
        long tiles = 0;
        for (size_t i = 0; i < n; ++i)
            if (pr.plan->items[i].n_rows > 0 && !by_copy_engine(ctx, pr.entry[i])) tiles += (pr.plan->items[i].n_rows + rpt - 1) / rpt;
        return tiles * n_layers;
    };
    auto busiest_cu_bytes = [&](int rpt) {
        const long tiles = tiles_with(rpt);
        const size_t tile_bytes = (size_t)rpt * rb;
        const long base = tiles / n_cu, rem = tiles % n_cu;          // CUs [0, rem) run one tile more
        const long eb = extra_wgs / n_cu, er = extra_wgs % n_cu;     // CUs [rem, rem + er) mod n_cu one extra workgroup more
        const size_t most_tiles = (size_t)(base + (rem > 0)) * tile_bytes + (size_t)eb * extra_bytes;
        const size_t most_extra = (size_t)base * tile_bytes + (size_t)(eb + (er > 0)) * extra_bytes;
        if (rem > 0 && rem + er > n_cu) return (size_t)(base + 1) * tile_bytes + (size_t)(eb + 1) * extra_bytes;   // a CU has both
        return std::max(most_tiles, most_extra);
    };
    int best = 0;
    size_t best_bytes = 0;
    for (const size_t kib : {32, 24, 16}) {
        const int rpt = std::max(1, (int)(kib * 1024 / rb));
        if (rpt == best) continue;
        const size_t bytes = busiest_cu_bytes(rpt);
        if (best == 0 || bytes < best_bytes) {
            best = rpt;
            best_bytes = bytes;
        }
    }
    return best;
}

int tiles_of(const GatherSeg &sg, int rows_per_tile)
{
    const int rpt = sg.src_k ? rows_per_tile : rows_per_tile * kPosOnlyTileFactor;
    return (sg.n_rows + rpt - 1) / rpt;
}

// Plan item i as a gather segment of this layer.  A module that the copy engine brings in is transferred here
// (one transfer per tensor on the caller's stream, straight into the packed rows: a module is contiguous on
// both sides) and left to the kernel for its position IDs only.
int segment_of(pc_ctx *ctx, const PlanRef &pr, size_t i, const int *kv_offsets, void *out_K, void *out_V,
               hipStream_t stream, GatherSeg &sg)
{
    const PlanItem &it = pr.plan->items[i];
    const ModuleEntry *m = pr.entry[i];
    const uint8_t *pool = m->host ? ctx->host_pool : ctx->pool;
    sg.src_k = pool + m->k_offset;
    sg.src_v = pool + m->v_offset;
    sg.dst_row = kv_offsets[it.prompt] + it.row;
    sg.n_rows = it.n_rows;
    sg.start_pos = it.start_pos;
    sg.first_tile = 0;
    if (by_copy_engine(ctx, m)) {
        const size_t bytes = (size_t)sg.n_rows * ctx->row_bytes, dst = (size_t)sg.dst_row * ctx->row_bytes;
        if (hipMemcpyAsync(static_cast<uint8_t *>(out_K) + dst, sg.src_k, bytes, hipMemcpyHostToDevice, stream) != hipSuccess ||
            hipMemcpyAsync(static_cast<uint8_t *>(out_V) + dst, sg.src_v, bytes, hipMemcpyHostToDevice, stream) != hipSuccess) {
            (void)hipGetLastError();
            return PC_E_HIP;
        }
        sg.src_k = sg.src_v = nullptr;
    }
    return PC_OK;
}

// Gather launches for a planned call: as many as the segment table of the kernel arguments needs
// (kMaxGatherSegs segments each); nothing is allocated.
int run_gather(pc_ctx *ctx, const PlanRef &pr, const int *kv_offsets, void *out_K, void *out_V, int32_t *out_pos,
               hipStream_t stream)
{
    const int rows_per_tile = gather_rows_per_tile(ctx, pr);
    const size_t n = pr.plan->items.size();
    size_t i = 0;
    while (i < n) {
        GatherArgs a;
        a.n_segs = 0;
        a.rows_per_tile = rows_per_tile;
        a.row_bytes = (int)ctx->row_bytes;
        int tiles = 0;
        for (; i < n && a.n_segs < kMaxGatherSegs; ++i) {
            if (pr.plan->items[i].n_rows == 0) continue;
            GatherSeg &sg = a.seg[a.n_segs];
            int rc = segment_of(ctx, pr, i, kv_offsets, out_K, out_V, stream, sg);
            if (rc != PC_OK) return rc;
            sg.first_tile = tiles;
            tiles += tiles_of(sg, rows_per_tile);
            ++a.n_segs;
        }
        a.total_tiles = tiles;
        if (a.n_segs == 0) break;
        int rc = launch_gather(ctx, a, static_cast<uint8_t *>(out_K), static_cast<uint8_t *>(out_V), out_pos, stream);
        if (rc != PC_OK) return rc;
    }
    return PC_OK;
}

int count_segments(const PlanRef &pr)
{
    int n = 0;
    for (const PlanItem &it : pr.plan->items) n += it.n_rows > 0;
    return n;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Factor folded into a pre-rotated Q: 1/sqrt(d), in the log2 domain for the bf16 kernels (their softmax is base 2).
float q_prescale(const pc_ctx *ctx)
{
    const float inv = 1.0f / sqrtf((float)ctx->cfg.head_dim);
    return ctx->cfg.dtype == PC_F32 ? inv : 1.4426950408889634f * inv;
}

int run_attn(pc_ctx *ctx, const AttnBatch &b, const void *Q, const int32_t *q_pos, const void *K, const void *V,
             const int32_t *pos, void *out, hipStream_t stream, bool q_rotated = false, const ScratchRef *scratch = nullptr)
{
    if (ctx->cfg.dtype == PC_F32)   // one wave per (query, head), no KV split: no scratch
        return launch_attn_f32(ctx, b, static_cast<const float *>(Q), q_pos, static_cast<const float *>(K),
                               static_cast<const float *>(V), pos, static_cast<float *>(out), stream, nullptr, q_rotated);
    return launch_attn_bf16(ctx, b, Q, q_pos, K, V, pos, out, stream, nullptr, q_rotated, scratch);
}

}  // namespace

extern "C" {

const char *pc_strerror(int status)
{
    switch (status) {
    case PC_OK: return "ok";
    case PC_E_BADARG: return "bad argument";
    case PC_E_LAYER: return "layer out of range";
    case PC_E_UNKNOWN_MODULE: return "module not stored for this layer";
    case PC_E_OVERLAP: return "selected modules overlap in position IDs";
    case PC_E_CAPACITY: return "output buffer or scratch too small";
    case PC_E_POOL_FULL: return "module pool exhausted";
    case PC_E_DUP_MODULE: return "module id already stored with another length or start position";
    case PC_E_POS_RANGE: return "position ID outside [0, max_pos)";
    case PC_E_UNSUPPORTED: return "unsupported head_dim / dtype";
    case PC_E_HIP: return "HIP runtime error";
    case PC_E_PARAM: return "no such parameter, or argument longer than the parameter";
    case PC_E_SCHEMA: return "malformed schema";
    default: return "unknown status";
    }
}

int pc_create(const pc_config *cfg, pc_ctx **out_ctx)
{
    if (!out_ctx) return PC_E_BADARG;
    *out_ctx = nullptr;
    int rc = validate_config(cfg);
    if (rc != PC_OK) return rc;

    pc_ctx *ctx = new (std::nothrow) pc_ctx();
    if (!ctx) return PC_E_HIP;
    ctx->cfg = *cfg;
    ctx->elem_bytes = elem_size(cfg->dtype);
    ctx->row_bytes = (size_t)cfg->n_kv_heads * cfg->head_dim * ctx->elem_bytes;
    ctx->modules.resize(cfg->n_layers);
    ctx->scratch_bytes = cfg->scratch_bytes ? cfg->scratch_bytes : kDefaultScratch;

    bool ok = hipGetDevice(&ctx->device) == hipSuccess && ctx->device >= 0 && ctx->device < kMaxDevices;
    if (ok && !g_static_scratch[ctx->device]) {   // this device's copy of the fixed scratch array
        void *ptr = nullptr;
        ok = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) == hipSuccess && ptr != nullptr;
        if (ok) g_static_scratch[ctx->device] = static_cast<uint8_t *>(ptr);
    }
    if (ok) ctx->static_scratch = g_static_scratch[ctx->device];
    hipDeviceProp_t prop;
    if (ok && hipGetDeviceProperties(&prop, ctx->device) == hipSuccess) ctx->n_cu = prop.multiProcessorCount;
    if (ok && cfg->pool_bytes) ok = hipMalloc(reinterpret_cast<void **>(&ctx->pool), cfg->pool_bytes) == hipSuccess;
    if (ok) ok = hipMalloc(reinterpret_cast<void **>(&ctx->scratch), ctx->scratch_bytes) == hipSuccess;

    // RoPE table: (cos, sin) of pos * base^(-2i/d), angles in fp64 (Sec. 4.2: a table looked up by position ID)
    const int half = cfg->head_dim / 2;
    const size_t n_entries = (size_t)cfg->max_pos * half;
    if (ok) ok = hipMalloc(reinterpret_cast<void **>(&ctx->rope_table), n_entries * sizeof(float2)) == hipSuccess;
    if (ok) {
        std::vector<float2> host(n_entries);
        std::vector<double> theta(half);
        for (int i = 0; i < half; ++i) theta[i] = pow(cfg->rope_base, -2.0 * (double)i / (double)cfg->head_dim);
        for (int p = 0; p < cfg->max_pos; ++p)
            for (int i = 0; i < half; ++i) {
                const double a = (double)p * theta[i];
                host[(size_t)p * half + i] = make_float2((float)cos(a), (float)sin(a));
            }
        ok = hipMemcpy(ctx->rope_table, host.data(), n_entries * sizeof(float2), hipMemcpyHostToDevice) == hipSuccess;
        // position-minor copy for the attention kernel whose lanes each hold one query (often consecutive positions)
        if (ok) ok = hipMalloc(reinterpret_cast<void **>(&ctx->rope_table_t), n_entries * sizeof(float2)) == hipSuccess;
        if (ok) {
            std::vector<float2> host_t(n_entries);
            for (int p = 0; p < cfg->max_pos; ++p)
                for (int i = 0; i < half; ++i) host_t[(size_t)i * cfg->max_pos + p] = host[(size_t)p * half + i];
            ok = hipMemcpy(ctx->rope_table_t, host_t.data(), n_entries * sizeof(float2), hipMemcpyHostToDevice) == hipSuccess;
        }
        if (ok) ok = hipMalloc(reinterpret_cast<void **>(&ctx->alibi), (size_t)cfg->n_q_heads * sizeof(float)) == hipSuccess;
        if (ok) ok = hipMalloc(reinterpret_cast<void **>(&ctx->iota), (size_t)cfg->max_pos * sizeof(int32_t)) == hipSuccess;
        if (ok) {
            std::vector<int32_t> ids(cfg->max_pos);
            for (int p = 0; p < cfg->max_pos; ++p) ids[p] = p;
            ok = hipMemcpy(ctx->iota, ids.data(), ids.size() * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess;
        }
    }
    if (!ok) {
        (void)hipGetLastError();
        if (ctx->pool) (void)hipFree(ctx->pool);
        if (ctx->scratch) (void)hipFree(ctx->scratch);
        if (ctx->rope_table) (void)hipFree(ctx->rope_table);
        if (ctx->rope_table_t) (void)hipFree(ctx->rope_table_t);
        if (ctx->iota) (void)hipFree(ctx->iota);
        if (ctx->alibi) (void)hipFree(ctx->alibi);
        delete ctx;
        return PC_E_HIP;
    }
    *out_ctx = ctx;
    return PC_OK;
}

static void free_profiler(pc_ctx *ctx)
{
    for (int k = 0; k < kProfKinds; ++k) {
        for (hipEvent_t e : ctx->prof.start[k]) (void)hipEventDestroy(e);
        for (hipEvent_t e : ctx->prof.stop[k]) (void)hipEventDestroy(e);
        ctx->prof.start[k].clear();
        ctx->prof.stop[k].clear();
        ctx->prof.used[k] = 0;
    }
    ctx->prof.capacity = 0;
}

int pc_profile_enable(pc_ctx *ctx, int max_records_per_kind)
{
    if (!ctx || max_records_per_kind < 0) return PC_E_BADARG;
    (void)hipDeviceSynchronize();
    free_profiler(ctx);
    for (int k = 0; k < kProfKinds; ++k)
        for (int i = 0; i < max_records_per_kind; ++i) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) { free_profiler(ctx); return PC_E_HIP; }
            if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); free_profiler(ctx); return PC_E_HIP; }
            ctx->prof.start[k].push_back(a);
            ctx->prof.stop[k].push_back(b);
        }
    ctx->prof.capacity = max_records_per_kind;
    return PC_OK;
}

int pc_profile_read_each(pc_ctx *ctx, int kind, float *ms_out, int capacity, int *n_records, double *total_ms)
{
    if (!ctx || kind < 0 || kind >= kProfKinds || capacity < 0 || (capacity > 0 && !ms_out)) return PC_E_BADARG;
    double sum = 0.0;
    const int n = ctx->prof.used[kind];
    for (int i = 0; i < n; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(ctx->prof.stop[kind][i]) != hipSuccess ||
            hipEventElapsedTime(&ms, ctx->prof.start[kind][i], ctx->prof.stop[kind][i]) != hipSuccess) {
            (void)hipGetLastError();
            return PC_E_HIP;
        }
        if (i < capacity) ms_out[i] = ms;
        sum += ms;
    }
    ctx->prof.used[kind] = 0;
    if (n_records) *n_records = n;
    if (total_ms) *total_ms = sum;
    return PC_OK;
}

int pc_profile_read(pc_ctx *ctx, int kind, int *n_records, double *total_ms)
{
    return pc_profile_read_each(ctx, kind, nullptr, 0, n_records, total_ms);
}

int pc_destroy(pc_ctx *ctx)
{
    if (!ctx) return PC_E_BADARG;
    (void)hipDeviceSynchronize();
    free_profiler(ctx);
    if (ctx->pool) (void)hipFree(ctx->pool);
    if (ctx->scratch) (void)hipFree(ctx->scratch);
    if (ctx->rope_table) (void)hipFree(ctx->rope_table);
    if (ctx->rope_table_t) (void)hipFree(ctx->rope_table_t);
    if (ctx->iota) (void)hipFree(ctx->iota);
    if (ctx->alibi) (void)hipFree(ctx->alibi);
    if (ctx->host_pool) (void)hipHostFree(ctx->host_pool);
    delete ctx;
    return PC_OK;
}

int pc_store_module(pc_ctx *ctx, int layer, int module_id, const void *K, const void *V, int n_tokens, int start_pos,
                    void *stream)
{
    if (!ctx || module_id < 0 || n_tokens < 0) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    if (n_tokens > 0 && (!K || !V)) return PC_E_BADARG;
    if (start_pos < 0 || (long)start_pos + n_tokens > (long)ctx->cfg.max_pos) return PC_E_POS_RANGE;

    auto &table = ctx->modules[layer];
    const size_t bytes = (size_t)n_tokens * ctx->row_bytes;
    auto it = table.find(module_id);
    ModuleEntry e;
    if (it != table.end()) {
        if (it->second.n_tokens != n_tokens || it->second.start_pos != start_pos || it->second.host) return PC_E_DUP_MODULE;
        e = it->second;  // refresh in place
    } else {
        const size_t k_off = align_up(ctx->pool_used, kPoolAlign);
        const size_t v_off = align_up(k_off + bytes, kPoolAlign);
        if (v_off + bytes > ctx->cfg.pool_bytes) return PC_E_POOL_FULL;
        e.k_offset = k_off;
        e.v_offset = v_off;
        e.n_tokens = n_tokens;
        e.start_pos = start_pos;
    }
    if (bytes) {
        if (hipMemcpyAsync(ctx->pool + e.k_offset, K, bytes, hipMemcpyDeviceToDevice, as_stream(stream)) != hipSuccess ||
            hipMemcpyAsync(ctx->pool + e.v_offset, V, bytes, hipMemcpyDeviceToDevice, as_stream(stream)) != hipSuccess) {
            (void)hipGetLastError();
            return PC_E_HIP;
        }
    }
    if (it == table.end()) {
        table.emplace(module_id, e);
        ctx->pool_used = e.v_offset + bytes;
        ++ctx->generation;   // cached plans were made without this module
    }
    return PC_OK;
}

int pc_resolve_scaffolds(int n_ids, const int *ids, int n_scaffolds, const int *scaffold_offsets, const int *member_ids,
                         const int *override_ids, int *out_ids)
{
    if (n_ids < 0 || n_scaffolds < 0 || (n_ids > 0 && (!ids || !out_ids))) return PC_E_BADARG;
    if (n_scaffolds > 0 && (!scaffold_offsets || !member_ids || !override_ids)) return PC_E_BADARG;
    std::vector<Scaffold> sc(n_scaffolds);
    for (int s = 0; s < n_scaffolds; ++s) {
        const int lo = scaffold_offsets[s], hi = scaffold_offsets[s + 1];
        if (lo < 0 || hi <= lo) return PC_E_BADARG;
        sc[s].member.assign(member_ids + lo, member_ids + hi);
        sc[s].override_id.assign(override_ids + lo, override_ids + hi);
    }
    cvec<int> v(ids, ids + n_ids);
    apply_scaffolds(sc, v);
    for (int i = 0; i < n_ids; ++i) out_ids[i] = v[i];
    return PC_OK;
}

int pc_define_scaffold(pc_ctx *ctx, int n_members, const int *member_ids, const int *override_ids)
{
    if (!ctx || n_members <= 0 || !member_ids || !override_ids) return PC_E_BADARG;
    Scaffold sc;
    for (int i = 0; i < n_members; ++i) {
        if (member_ids[i] < 0 || override_ids[i] < 0) return PC_E_BADARG;
        for (int j = 0; j < i; ++j)
            if (member_ids[j] == member_ids[i]) return PC_E_BADARG;
        sc.member.push_back(member_ids[i]);
        sc.override_id.push_back(override_ids[i]);
    }
    ctx->scaffolds.push_back(sc);
    ++ctx->generation;   // cached plans were made without this scaffold
    return PC_OK;
}

int pc_alibi_slopes(int n_heads, float *slopes)
{
    if (n_heads <= 0 || !slopes) return PC_E_BADARG;
    // largest power of two not above n_heads gets the sequence 2^(-8 i / p), i = 1..p; the remaining
    // heads take the odd members of the sequence for 2p
    int p = 1;
    while (p * 2 <= n_heads) p *= 2;
    for (int h = 0; h < n_heads; ++h) {
        const double e = h < p ? 8.0 * (h + 1) / p : 4.0 * (2 * (h - p) + 1) / p;
        slopes[h] = (float)exp2(-e);
    }
    return PC_OK;
}

int pc_set_alibi(pc_ctx *ctx, const float *slopes)
{
    if (!ctx) return PC_E_BADARG;
    if (!slopes) {
        ctx->use_alibi = false;
        return PC_OK;
    }
    for (int h = 0; h < ctx->cfg.n_q_heads; ++h)
        if (!(slopes[h] >= 0.f) || !std::isfinite(slopes[h])) return PC_E_BADARG;
    if (hipSetDevice(ctx->device) != hipSuccess ||
        hipMemcpy(ctx->alibi, slopes, (size_t)ctx->cfg.n_q_heads * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        return PC_E_HIP;
    }
    ctx->use_alibi = true;
    return PC_OK;
}

int pc_host_pool_reserve(pc_ctx *ctx, size_t bytes)
{
    if (!ctx || bytes == 0 || ctx->host_pool) return PC_E_BADARG;
    if (hipSetDevice(ctx->device) != hipSuccess) return PC_E_HIP;
    void *p = nullptr;
    // pinned and mapped: the copy engine transfers from it at link speed and kernels can load from it
    if (hipHostMalloc(&p, bytes, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        return PC_E_HIP;
    }
    ctx->host_pool = static_cast<uint8_t *>(p);
    ctx->host_pool_bytes = bytes;
    ctx->host_pool_used = 0;
    return PC_OK;
}

int pc_set_host_copy_mode(pc_ctx *ctx, int mode)
{
    if (!ctx || (mode != PC_HOST_READ_KERNEL && mode != PC_HOST_COPY_ENGINE)) return PC_E_BADARG;
    ctx->host_copy_mode = mode;
    return PC_OK;
}

int pc_set_attn_kernel(pc_ctx *ctx, int which)
{
    if (!ctx || (which != PC_ATTN_AUTO && which != PC_ATTN_REGISTER_STAGED)) return PC_E_BADARG;
    ctx->attn_kernel = which;
    return PC_OK;
}

int pc_store_module_host(pc_ctx *ctx, int layer, int module_id, const void *K_host, const void *V_host, int n_tokens,
                         int start_pos)
{
    if (!ctx || module_id < 0 || n_tokens < 0) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    if (n_tokens > 0 && (!K_host || !V_host)) return PC_E_BADARG;
    if (start_pos < 0 || (long)start_pos + n_tokens > (long)ctx->cfg.max_pos) return PC_E_POS_RANGE;

    auto &table = ctx->modules[layer];
    const size_t bytes = (size_t)n_tokens * ctx->row_bytes;
    auto it = table.find(module_id);
    ModuleEntry e;
    if (it != table.end()) {
        // refresh in place; a module keeps the tier it was first stored in
        if (it->second.n_tokens != n_tokens || it->second.start_pos != start_pos || !it->second.host) return PC_E_DUP_MODULE;
        e = it->second;
    } else {
        const size_t k_off = align_up(ctx->host_pool_used, kPoolAlign);
        const size_t v_off = align_up(k_off + bytes, kPoolAlign);
        if (!ctx->host_pool || v_off + bytes > ctx->host_pool_bytes) return PC_E_POOL_FULL;
        e.k_offset = k_off;
        e.v_offset = v_off;
        e.n_tokens = n_tokens;
        e.start_pos = start_pos;
        e.host = true;
    }
    if (bytes) {
        memcpy(ctx->host_pool + e.k_offset, K_host, bytes);
        memcpy(ctx->host_pool + e.v_offset, V_host, bytes);
    }
    if (it == table.end()) {
        table.emplace(module_id, e);
        ctx->host_pool_used = e.v_offset + bytes;
        ++ctx->generation;
    }
    return PC_OK;
}

int pc_assemble_kv(pc_ctx *ctx, int layer, const int *module_ids, int n_modules, void *out_K, void *out_V,
                   int32_t *out_pos, int capacity_tokens, int *out_n_tokens, void *stream)
{
    if (!ctx || n_modules < 0 || capacity_tokens < 0 || (n_modules > 0 && !module_ids)) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    if (!out_K || !out_V || !out_pos || !aligned16(out_K) || !aligned16(out_V)) return PC_E_BADARG;
    const int mod_offsets[2] = {0, n_modules}, kv_offsets[2] = {0, capacity_tokens};
    PlanRef pr;
    int rc = get_plan(ctx, layer, module_ids, mod_offsets, 1, kv_offsets, nullptr, pr);
    if (rc != PC_OK) return rc;
    rc = run_gather(ctx, pr, kv_offsets, out_K, out_V, out_pos, as_stream(stream));
    if (rc == PC_OK && out_n_tokens) *out_n_tokens = pr.plan->prompt_rows[0];
    return rc;
}

int pc_assemble_kv_batched(pc_ctx *ctx, int layer, const int *module_ids_flat, const int *mod_offsets, int n_prompts,
                           void *out_K, void *out_V, int32_t *out_pos, const int *kv_offsets, int *out_n_tokens,
                           void *stream)
{
    if (!ctx || n_prompts < 0 || !mod_offsets || !kv_offsets) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    if (!out_K || !out_V || !out_pos || !aligned16(out_K) || !aligned16(out_V)) return PC_E_BADARG;
    for (int b = 0; b < n_prompts; ++b)
        if (kv_offsets[b + 1] - kv_offsets[b] < 0 || kv_offsets[b] < 0) return PC_E_BADARG;
    PlanRef pr;
    int rc = get_plan(ctx, layer, module_ids_flat, mod_offsets, n_prompts, kv_offsets, nullptr, pr);
    if (rc != PC_OK) return rc;
    rc = run_gather(ctx, pr, kv_offsets, out_K, out_V, out_pos, as_stream(stream));
    if (rc == PC_OK && out_n_tokens)
        for (int b = 0; b < n_prompts; ++b) out_n_tokens[b] = pr.plan->prompt_rows[b];
    return rc;
}

int pc_assemble_kv_layers(pc_ctx *ctx, int first_layer, int n_layers, const int *module_ids_flat, const int *mod_offsets,
                          int n_prompts, void *const *out_K, void *const *out_V, int32_t *const *out_pos,
                          const int *kv_offsets, int *out_n_tokens, void *stream)
{
    if (!ctx || n_prompts < 0 || n_layers < 0 || !mod_offsets || !kv_offsets) return PC_E_BADARG;
    if (first_layer < 0 || (long)first_layer + n_layers > (long)ctx->cfg.n_layers) return PC_E_LAYER;
    if (n_layers > 0 && (!out_K || !out_V || !out_pos)) return PC_E_BADARG;
    for (int l = 0; l < n_layers; ++l)
        if (!out_K[l] || !out_V[l] || !out_pos[l] || !aligned16(out_K[l]) || !aligned16(out_V[l])) return PC_E_BADARG;
    for (int b = 0; b < n_prompts; ++b)
        if (kv_offsets[b + 1] - kv_offsets[b] < 0 || kv_offsets[b] < 0) return PC_E_BADARG;
    // every layer is planned (validated) before the first launch: an error leaves all outputs untouched
    PlanRef first;
    int segs_per_layer = 0;   // of the layer with most
    for (int l = 0; l < n_layers; ++l) {
        PlanRef pr;
        int rc = get_plan(ctx, first_layer + l, module_ids_flat, mod_offsets, n_prompts, kv_offsets, nullptr, pr);
        if (rc != PC_OK) return rc;
        if (l == 0) first = pr;
        segs_per_layer = std::max(segs_per_layer, count_segments(pr));
    }
    if (n_layers == 0) return PC_OK;
    hipStream_t st = as_stream(stream);
    if (segs_per_layer > kMaxGatherSegs) {   // more segments per layer than one launch holds: layer by layer
        for (int l = 0; l < n_layers; ++l) {
            PlanRef pr;
            int rc = get_plan(ctx, first_layer + l, module_ids_flat, mod_offsets, n_prompts, kv_offsets, nullptr, pr);
            if (rc == PC_OK) rc = run_gather(ctx, pr, kv_offsets, out_K[l], out_V[l], out_pos[l], st);
            if (rc != PC_OK) return rc;
        }
    } else if (segs_per_layer > 0) {
        const int layers_per_launch = std::min(kMaxGatherLayers, kMaxGatherSegs / segs_per_layer);
        for (int l0 = 0; l0 < n_layers; l0 += layers_per_launch) {
            const int nl = std::min(layers_per_launch, n_layers - l0);
            GatherLayersArgs a;
            a.g.n_segs = 0;
            a.g.row_bytes = (int)ctx->row_bytes;
            int tiles = 0;
            for (int l = 0; l < nl; ++l) {
                PlanRef pr;   // a cache hit (planned above); a layer that differs from the first one has a plan of its own
                int rc = get_plan(ctx, first_layer + l0 + l, module_ids_flat, mod_offsets, n_prompts, kv_offsets, nullptr, pr);
                if (rc != PC_OK) return rc;
                if (l == 0) a.g.rows_per_tile = gather_rows_per_tile(ctx, pr, 0, nl);
                a.out[l] = GatherLayerOut{static_cast<uint8_t *>(out_K[l0 + l]), static_cast<uint8_t *>(out_V[l0 + l]), out_pos[l0 + l]};
                for (size_t i = 0; i < pr.plan->items.size(); ++i) {
                    if (pr.plan->items[i].n_rows == 0) continue;
                    GatherSeg &sg = a.g.seg[a.g.n_segs];
                    rc = segment_of(ctx, pr, i, kv_offsets, out_K[l0 + l], out_V[l0 + l], st, sg);
                    if (rc != PC_OK) return rc;
                    sg.first_tile = tiles;
                    tiles += tiles_of(sg, a.g.rows_per_tile);
                    a.seg_layer[a.g.n_segs] = (unsigned char)l;
                    ++a.g.n_segs;
                }
            }
            a.g.total_tiles = tiles;
            int rc = launch_gather_layers(ctx, a, st);
            if (rc != PC_OK) return rc;
        }
    }
    if (out_n_tokens)
        for (int b = 0; b < n_prompts; ++b) out_n_tokens[b] = first.plan->prompt_rows[b];
    return PC_OK;
}

int pc_rope(pc_ctx *ctx, void *x, int n_tokens, int n_heads, const int32_t *pos, void *stream)
{
    if (!ctx || n_tokens < 0 || n_heads <= 0) return PC_E_BADARG;
    if (n_tokens == 0) return PC_OK;
    if (!x || !pos) return PC_E_BADARG;
    return launch_rope(ctx, x, n_tokens, n_heads, pos, as_stream(stream));
}

static int append_impl(pc_ctx *ctx, int layer, const void *K_new_raw, const void *V_new, const int32_t *q_pos,
                       const int *q_offsets, int n_prompts, void *asm_K, void *asm_V, int32_t *asm_pos,
                       const int *kv_offsets, const int *kv_lens, void *stream, const void *Q_new, void *Q_rot)
{
    if (!ctx || n_prompts < 0 || !q_offsets || !kv_offsets || !kv_lens) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    for (int b = 0; b < n_prompts; ++b) {
        const int n = q_offsets[b + 1] - q_offsets[b];
        if (n < 0 || kv_lens[b] < 0 || q_offsets[b] < 0 || kv_offsets[b] < 0) return PC_E_BADARG;
        if ((long)kv_offsets[b] + kv_lens[b] + n > (long)kv_offsets[b + 1]) return PC_E_CAPACITY;
    }
    if (n_prompts > 0 && q_offsets[n_prompts] > q_offsets[0] && (!K_new_raw || !V_new || !q_pos || !asm_K || !asm_V || !asm_pos))
        return PC_E_BADARG;
    for (int base = 0; base < n_prompts; base += kMaxAppendSegs) {
        AppendArgs a;
        a.n_segs = std::min(kMaxAppendSegs, n_prompts - base);
        a.total_rows = 0;
        for (int i = 0; i < a.n_segs; ++i) {
            const int b = base + i;
            a.seg[i].q_begin = q_offsets[b];
            a.seg[i].n = q_offsets[b + 1] - q_offsets[b];
            a.seg[i].dst_row = kv_offsets[b] + kv_lens[b];
            a.seg[i].pos0 = kPosFromArray;
            a.total_rows += a.seg[i].n;
        }
        int rc = launch_append(ctx, a, K_new_raw, V_new, q_pos, asm_K, asm_V, asm_pos, as_stream(stream), Q_new, Q_rot,
                               q_prescale(ctx));
        if (rc != PC_OK) return rc;
    }
    return PC_OK;
}

int pc_append_kv_batched(pc_ctx *ctx, int layer, const void *K_new_raw, const void *V_new, const int32_t *q_pos,
                         const int *q_offsets, int n_prompts, void *asm_K, void *asm_V, int32_t *asm_pos,
                         const int *kv_offsets, const int *kv_lens, void *stream)
{
    return append_impl(ctx, layer, K_new_raw, V_new, q_pos, q_offsets, n_prompts, asm_K, asm_V, asm_pos, kv_offsets, kv_lens,
                       stream, nullptr, nullptr);
}

int pc_append_rotate_batched(pc_ctx *ctx, int layer, const void *K_new_raw, const void *V_new, const void *Q_new,
                             const int32_t *q_pos, const int *q_offsets, int n_prompts, void *asm_K, void *asm_V,
                             int32_t *asm_pos, const int *kv_offsets, const int *kv_lens, void *Q_rot, void *stream)
{
    if (!ctx || n_prompts < 0 || !q_offsets) return PC_E_BADARG;
    if (n_prompts > 0 && q_offsets[n_prompts] > q_offsets[0] && (!Q_new || !Q_rot || !aligned16(Q_new) || !aligned16(Q_rot)))
        return PC_E_BADARG;
    return append_impl(ctx, layer, K_new_raw, V_new, q_pos, q_offsets, n_prompts, asm_K, asm_V, asm_pos, kv_offsets, kv_lens,
                       stream, Q_new, Q_rot);
}

static int assemble_append_impl(pc_ctx *ctx, int layer, const int *module_ids_flat, const int *mod_offsets,
                                int n_prompts, const void *K_new_raw, const void *V_new, const int32_t *q_pos,
                                const int *q_offsets, void *out_K, void *out_V, int32_t *out_pos,
                                const int *kv_offsets, int *out_n_tokens, void *stream, const void *Q_new, void *Q_rot)
{
    if (!ctx || n_prompts < 0 || !mod_offsets || !kv_offsets || !q_offsets) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    if (!out_K || !out_V || !out_pos || !aligned16(out_K) || !aligned16(out_V)) return PC_E_BADARG;
    long new_rows = 0;
    for (int b = 0; b < n_prompts; ++b) {
        const int cap = kv_offsets[b + 1] - kv_offsets[b];
        const int nq = q_offsets[b + 1] - q_offsets[b];
        if (cap < 0 || nq < 0 || kv_offsets[b] < 0 || q_offsets[b] < 0) return PC_E_BADARG;
        new_rows += nq;
    }
    PlanRef pr;
    int rc = get_plan(ctx, layer, module_ids_flat, mod_offsets, n_prompts, kv_offsets, q_offsets, pr);
    if (rc != PC_OK) return rc;
    if (new_rows > 0 && (!K_new_raw || !V_new || !q_pos)) return PC_E_BADARG;
    const int *rows = pr.plan->prompt_rows.data();

    const int n_segs = count_segments(pr);
    if (n_segs <= kMaxGatherSegs && n_prompts <= kMaxFusedAppendSegs) {
        FusedKvArgs a;
        // an appended row's workgroup moves the token's K and V rows and, when it rotates Q as well, its Q row
        const size_t app_bytes = ctx->row_bytes + (Q_rot ? (size_t)ctx->cfg.n_q_heads * ctx->cfg.head_dim * ctx->elem_bytes / 2 : 0);
        const int rows_per_tile = gather_rows_per_tile(ctx, pr, new_rows, 1, app_bytes);
        a.g.n_segs = 0;
        a.g.rows_per_tile = rows_per_tile;
        a.g.row_bytes = (int)ctx->row_bytes;
        int tiles = 0;
        for (size_t i = 0; i < pr.plan->items.size(); ++i) {
            if (pr.plan->items[i].n_rows == 0) continue;
            GatherSeg &sg = a.g.seg[a.g.n_segs];
            rc = segment_of(ctx, pr, i, kv_offsets, out_K, out_V, as_stream(stream), sg);
            if (rc != PC_OK) return rc;
            sg.first_tile = tiles;
            tiles += tiles_of(sg, rows_per_tile);
            ++a.g.n_segs;
        }
        a.g.total_tiles = tiles;
        a.n_app = n_prompts;
        a.app_rows = (int)new_rows;
        for (int b = 0; b < n_prompts; ++b) {
            a.app[b].q_begin = q_offsets[b];
            a.app[b].n = q_offsets[b + 1] - q_offsets[b];
            a.app[b].dst_row = kv_offsets[b] + rows[b];
            a.app[b].pos0 = kPosFromArray;
        }
        rc = launch_gather_append(ctx, a, static_cast<uint8_t *>(out_K), static_cast<uint8_t *>(out_V), out_pos,
                                  K_new_raw, V_new, q_pos, as_stream(stream), Q_new, Q_rot, q_prescale(ctx));
    } else {
        // too many segments for one argument block: the two steps one after the other
        rc = run_gather(ctx, pr, kv_offsets, out_K, out_V, out_pos, as_stream(stream));
        if (rc == PC_OK)
            rc = append_impl(ctx, layer, K_new_raw, V_new, q_pos, q_offsets, n_prompts, out_K, out_V, out_pos, kv_offsets,
                             rows, stream, Q_new, Q_rot);
    }
    if (rc == PC_OK && out_n_tokens)
        for (int b = 0; b < n_prompts; ++b) out_n_tokens[b] = rows[b] + (q_offsets[b + 1] - q_offsets[b]);
    return rc;
}

int pc_assemble_append_kv_batched(pc_ctx *ctx, int layer, const int *module_ids_flat, const int *mod_offsets,
                                  int n_prompts, const void *K_new_raw, const void *V_new, const int32_t *q_pos,
                                  const int *q_offsets, void *out_K, void *out_V, int32_t *out_pos,
                                  const int *kv_offsets, int *out_n_tokens, void *stream)
{
    return assemble_append_impl(ctx, layer, module_ids_flat, mod_offsets, n_prompts, K_new_raw, V_new, q_pos, q_offsets, out_K,
                                out_V, out_pos, kv_offsets, out_n_tokens, stream, nullptr, nullptr);
}

int pc_assemble_append_rotate_batched(pc_ctx *ctx, int layer, const int *module_ids_flat, const int *mod_offsets,
                                      int n_prompts, const void *K_new_raw, const void *V_new, const void *Q_new,
                                      const int32_t *q_pos, const int *q_offsets, void *out_K, void *out_V,
                                      int32_t *out_pos, const int *kv_offsets, int *out_n_tokens, void *Q_rot, void *stream)
{
    if (!ctx || n_prompts < 0 || !q_offsets) return PC_E_BADARG;
    if (n_prompts > 0 && q_offsets[n_prompts] > q_offsets[0] && (!Q_new || !Q_rot || !aligned16(Q_new) || !aligned16(Q_rot)))
        return PC_E_BADARG;
    return assemble_append_impl(ctx, layer, module_ids_flat, mod_offsets, n_prompts, K_new_raw, V_new, q_pos, q_offsets, out_K,
                                out_V, out_pos, kv_offsets, out_n_tokens, stream, Q_new, Q_rot);
}

int pc_set_module_params(pc_ctx *ctx, int module_id, int n_params, const int *offsets, const int *lens)
{
    if (!ctx || n_params < 0 || (n_params > 0 && (!offsets || !lens))) return PC_E_BADARG;
    std::vector<ParamSlot> slots(n_params);
    long end = 0;
    for (int j = 0; j < n_params; ++j) {
        if (offsets[j] < end || lens[j] < 0) return PC_E_BADARG;   // sorted, disjoint, non-negative
        slots[j].offset = offsets[j];
        slots[j].len = lens[j];
        end = (long)offsets[j] + lens[j];
        if (end > ctx->cfg.max_pos) return PC_E_BADARG;
    }
    if (n_params == 0) ctx->params.erase(module_id);
    else ctx->params[module_id] = std::move(slots);
    return PC_OK;
}

int pc_fill_params(pc_ctx *ctx, int layer, const int *module_ids, int n_modules, int n_args, const int *arg_module,
                   const int *arg_param, const int *arg_offsets, const void *K_arg_raw, const void *V_arg, void *asm_K,
                   void *asm_V, int32_t *asm_pos, int capacity_tokens, void *stream)
{
    if (!ctx || n_modules < 0 || n_args < 0 || capacity_tokens < 0) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    if (n_modules > 0 && !module_ids) return PC_E_BADARG;
    if (n_args == 0) return PC_OK;
    if (!arg_module || !arg_param || !arg_offsets || !asm_K || !asm_V || !asm_pos) return PC_E_BADARG;
    // where each module's rows are in the packed buffer (the order pc_assemble_kv used)
    const auto &table = ctx->modules[layer];
    std::vector<int> row0(n_modules), len(n_modules), start(n_modules);
    long rows = 0;
    for (int i = 0; i < n_modules; ++i) {
        auto it = table.find(module_ids[i]);
        if (it == table.end()) return PC_E_UNKNOWN_MODULE;
        row0[i] = (int)rows;
        len[i] = it->second.n_tokens;
        start[i] = it->second.start_pos;
        rows += len[i];
    }
    if (rows > capacity_tokens) return PC_E_CAPACITY;
    std::vector<AppendSeg> segs;
    long total_arg_rows = 0;
    for (int a = 0; a < n_args; ++a) {
        const int mi = arg_module[a], n = arg_offsets[a + 1] - arg_offsets[a];
        if (mi < 0 || mi >= n_modules || n < 0 || arg_offsets[a] < 0) return PC_E_BADARG;
        auto ps = ctx->params.find(module_ids[mi]);
        if (ps == ctx->params.end() || arg_param[a] < 0 || arg_param[a] >= (int)ps->second.size()) return PC_E_PARAM;
        const ParamSlot slot = ps->second[arg_param[a]];
        if ((long)slot.offset + slot.len > len[mi] || n > slot.len) return PC_E_PARAM;
        if (n > 0) segs.push_back(AppendSeg{arg_offsets[a], n, row0[mi] + slot.offset, start[mi] + slot.offset});
        if (slot.len > n) segs.push_back(AppendSeg{0, slot.len - n, row0[mi] + slot.offset + n, kPosMaskRows});
        total_arg_rows += n;
    }
    if (total_arg_rows > 0 && (!K_arg_raw || !V_arg)) return PC_E_BADARG;
    for (size_t base = 0; base < segs.size(); base += kMaxAppendSegs) {
        AppendArgs a;
        a.n_segs = (int)std::min<size_t>(kMaxAppendSegs, segs.size() - base);
        a.total_rows = 0;
        for (int i = 0; i < a.n_segs; ++i) {
            a.seg[i] = segs[base + i];
            a.total_rows += a.seg[i].n;
        }
        int rc = launch_append(ctx, a, K_arg_raw, V_arg, nullptr, asm_K, asm_V, asm_pos, as_stream(stream));
        if (rc != PC_OK) return rc;
    }
    return PC_OK;
}

int pc_append_kv(pc_ctx *ctx, int layer, const void *K_new_raw, const void *V_new, const int32_t *q_pos, int n_q,
                 void *asm_K, void *asm_V, int32_t *asm_pos, int n_kv_before, int capacity_tokens, void *stream)
{
    if (n_q < 0 || n_kv_before < 0 || capacity_tokens < 0) return PC_E_BADARG;
    const int q_offsets[2] = {0, n_q};
    const int kv_offsets[2] = {0, capacity_tokens};
    const int kv_lens[1] = {n_kv_before};
    return pc_append_kv_batched(ctx, layer, K_new_raw, V_new, q_pos, q_offsets, 1, asm_K, asm_V, asm_pos, kv_offsets,
                                kv_lens, stream);
}

static int prefill_attn_batched_impl(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos, const int *q_offsets,
                                     int n_prompts, const void *asm_K, const void *asm_V, const int32_t *asm_pos,
                                     const int *kv_offsets, const int *kv_lens, void *out, void *stream, bool q_rotated,
                                     const ScratchRef *scratch = nullptr)
{
    if (!ctx || n_prompts < 0 || !q_offsets || !kv_offsets || !kv_lens) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    long total_q = 0;
    for (int b = 0; b < n_prompts; ++b) {
        const int n = q_offsets[b + 1] - q_offsets[b];
        if (n < 0 || kv_lens[b] < 0 || q_offsets[b] < 0 || kv_offsets[b] < 0) return PC_E_BADARG;
        total_q += n;
    }
    if (total_q == 0) return PC_OK;
    if (!Q_new || !q_pos || !out || !aligned16(Q_new) || !aligned16(out)) return PC_E_BADARG;
    bool any_kv = false;
    for (int b = 0; b < n_prompts; ++b) any_kv |= kv_lens[b] > 0;
    if (any_kv && (!asm_K || !asm_V || !asm_pos || !aligned16(asm_K) || !aligned16(asm_V))) return PC_E_BADARG;

    for (int base = 0; base < n_prompts; base += kMaxAttnSeqs) {
        AttnBatch ab;
        ab.n_seqs = std::min(kMaxAttnSeqs, n_prompts - base);
        for (int i = 0; i < ab.n_seqs; ++i) {
            const int b = base + i;
            ab.seq[i].q_begin = q_offsets[b];
            ab.seq[i].n_q = q_offsets[b + 1] - q_offsets[b];
            ab.seq[i].kv_begin = kv_offsets[b];
            ab.seq[i].n_kv = kv_lens[b];
        }
        int rc = run_attn(ctx, ab, Q_new, q_pos, asm_K, asm_V, asm_pos, out, as_stream(stream), q_rotated, scratch);
        if (rc != PC_OK) return rc;
    }
    return PC_OK;
}

int pc_prefill_attn_batched(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos, const int *q_offsets,
                            int n_prompts, const void *asm_K, const void *asm_V, const int32_t *asm_pos,
                            const int *kv_offsets, const int *kv_lens, void *out, void *stream)
{
    return prefill_attn_batched_impl(ctx, layer, Q_new, q_pos, q_offsets, n_prompts, asm_K, asm_V, asm_pos, kv_offsets, kv_lens,
                                     out, stream, false);
}

int pc_prefill_attn_rotated_batched(pc_ctx *ctx, int layer, const void *Q_rot, const int32_t *q_pos, const int *q_offsets,
                                    int n_prompts, const void *asm_K, const void *asm_V, const int32_t *asm_pos,
                                    const int *kv_offsets, const int *kv_lens, void *out, void *stream)
{
    return prefill_attn_batched_impl(ctx, layer, Q_rot, q_pos, q_offsets, n_prompts, asm_K, asm_V, asm_pos, kv_offsets, kv_lens,
                                     out, stream, true);
}

static int prefill_attn_shared_impl(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos, const int *q_offsets,
                                    int n_prompts, const int *module_ids_flat, const int *mod_offsets, const void *K_tail,
                                    const void *V_tail, void *out, void *stream, bool q_rotated);

int pc_prefill_attn_shared_batched(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos, const int *q_offsets,
                                   int n_prompts, const int *module_ids_flat, const int *mod_offsets, const void *K_tail,
                                   const void *V_tail, void *out, void *stream)
{
    return prefill_attn_shared_impl(ctx, layer, Q_new, q_pos, q_offsets, n_prompts, module_ids_flat, mod_offsets, K_tail, V_tail,
                                    out, stream, false);
}

int pc_prefill_attn_shared_rotated_batched(pc_ctx *ctx, int layer, const void *Q_rot, const int32_t *q_pos,
                                           const int *q_offsets, int n_prompts, const int *module_ids_flat,
                                           const int *mod_offsets, const void *K_tail, const void *V_tail, void *out,
                                           void *stream)
{
    return prefill_attn_shared_impl(ctx, layer, Q_rot, q_pos, q_offsets, n_prompts, module_ids_flat, mod_offsets, K_tail, V_tail,
                                    out, stream, true);
}

static int prefill_attn_shared_impl(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos, const int *q_offsets,
                                    int n_prompts, const int *module_ids_flat, const int *mod_offsets, const void *K_tail,
                                    const void *V_tail, void *out, void *stream, bool q_rotated)
{
    if (!ctx || n_prompts < 0 || !q_offsets || !mod_offsets) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    long total_q = 0;
    for (int b = 0; b < n_prompts; ++b) {
        const int n = q_offsets[b + 1] - q_offsets[b], nm = mod_offsets[b + 1] - mod_offsets[b];
        if (n < 0 || nm < 0 || q_offsets[b] < 0 || (nm > 0 && !module_ids_flat)) return PC_E_BADARG;
        total_q += n;
    }
    if (total_q == 0) return PC_OK;
    if (!Q_new || !q_pos || !out || !K_tail || !V_tail || !aligned16(Q_new) || !aligned16(out) || !aligned16(K_tail) ||
        !aligned16(V_tail))
        return PC_E_BADARG;
    const uint8_t *kt = static_cast<const uint8_t *>(K_tail), *vt = static_cast<const uint8_t *>(V_tail);
    // every prompt is checked before the first launch, so that an error leaves `out` untouched
    for (int b = 0; b < n_prompts; ++b) {
        const int nm = mod_offsets[b + 1] - mod_offsets[b], nq = q_offsets[b + 1] - q_offsets[b];
        if (nm + 1 > kMaxKvSegs || (size_t)nq * ctx->row_bytes >= ((size_t)1 << 32)) return PC_E_UNSUPPORTED;
    }
    PlanRef pr;
    int prc = get_plan(ctx, layer, module_ids_flat, mod_offsets, n_prompts, nullptr, nullptr, pr);
    if (prc != PC_OK) return prc;
    const size_t n_items = pr.plan->items.size();
    for (size_t i = 0; i < n_items; ++i) {
        if ((size_t)pr.plan->items[i].n_rows * ctx->row_bytes >= ((size_t)1 << 32)) return PC_E_UNSUPPORTED;   // 32-bit offsets inside a range
        if (pr.entry[i]->host) return PC_E_UNSUPPORTED;   // host-resident modules are assembled (copied), not read in place
    }
    int b = 0;
    size_t item = 0;   // first plan item of prompt b (items are grouped by prompt, in order)
    while (b < n_prompts) {
        // as many prompts per launch as the range table and the prompt table hold
        AttnBatch ab;
        KvSegTable tab;
        ab.n_seqs = 0;
        int n_seg = 0;
        for (; b < n_prompts && ab.n_seqs < kMaxAttnSeqs; ++b) {
            const int nm = mod_offsets[b + 1] - mod_offsets[b], nq = q_offsets[b + 1] - q_offsets[b];
            if (n_seg + nm + 1 > kMaxKvSegs) break;
            const int seg0 = n_seg;
            int rows = 0;
            for (; item < n_items && pr.plan->items[item].prompt == b; ++item) {
                const PlanItem &it = pr.plan->items[item];
                if (it.n_rows == 0) continue;
                const ModuleEntry *m = pr.entry[item];
                tab.seg[n_seg++] = KvSeg{ctx->pool + m->k_offset, ctx->pool + m->v_offset, ctx->iota + it.start_pos, rows, 0};
                rows += it.n_rows;
            }
            if (nq > 0) {   // the prompt's own tokens: rows q_offsets[b].. of the tail buffers, positions q_pos
                tab.seg[n_seg++] = KvSeg{kt + (size_t)q_offsets[b] * ctx->row_bytes, vt + (size_t)q_offsets[b] * ctx->row_bytes,
                                         q_pos + q_offsets[b], rows, 0};
                rows += nq;
            }
            tab.seg_begin[ab.n_seqs] = seg0;
            ab.seq[ab.n_seqs] = AttnSeq{q_offsets[b], nq, 0, rows};
            ++ab.n_seqs;
        }
        tab.seg_begin[ab.n_seqs] = n_seg;
        int rc = ctx->cfg.dtype == PC_F32
                     ? launch_attn_f32(ctx, ab, static_cast<const float *>(Q_new), q_pos, nullptr, nullptr, nullptr,
                                       static_cast<float *>(out), as_stream(stream), &tab, q_rotated)
                     : launch_attn_bf16(ctx, ab, Q_new, q_pos, nullptr, nullptr, nullptr, out, as_stream(stream), &tab,
                                        q_rotated);
        if (rc != PC_OK) return rc;
    }
    return PC_OK;
}

int pc_prefill_attn(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos, int n_q, const void *asm_K,
                    const void *asm_V, const int32_t *asm_pos, int n_kv, void *out, void *stream)
{
    if (n_q < 0 || n_kv < 0) return PC_E_BADARG;
    const int q_offsets[2] = {0, n_q};
    const int kv_offsets[2] = {0, n_kv};
    const int kv_lens[1] = {n_kv};
    return pc_prefill_attn_batched(ctx, layer, Q_new, q_pos, q_offsets, 1, asm_K, asm_V, asm_pos, kv_offsets, kv_lens,
                                   out, stream);
}

int pc_prefill_attn_static(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos, int n_q, const void *asm_K,
                           const void *asm_V, const int32_t *asm_pos, int n_kv, void *out, void *stream)
{
    if (!ctx || n_q < 0 || n_kv < 0) return PC_E_BADARG;
    if (!ctx->static_scratch) return PC_E_HIP;
    const int q_offsets[2] = {0, n_q};
    const int kv_offsets[2] = {0, n_kv};
    const int kv_lens[1] = {n_kv};
    const ScratchRef fixed{ctx->static_scratch, kStaticScratchBytes, true};
    return prefill_attn_batched_impl(ctx, layer, Q_new, q_pos, q_offsets, 1, asm_K, asm_V, asm_pos, kv_offsets, kv_lens, out,
                                     stream, false, &fixed);
}

int pc_plan_stats(const pc_ctx *ctx, long *hits, long *misses, long *heap_allocs)
{
    if (!ctx) return PC_E_BADARG;
    if (hits) *hits = (long)ctx->plan_hits;
    if (misses) *misses = (long)ctx->plan_misses;
    if (heap_allocs) *heap_allocs = g_plan_heap_allocs;
    return PC_OK;
}

/* ------------------------------------------------------------ host integers */

long pc_schema_layout(int n, const int *sizes, const int *union_ids, int *starts)
{
    if (n < 0 || (n > 0 && (!sizes || !union_ids || !starts))) return PC_E_SCHEMA;
    // a union's children must form one contiguous run
    std::vector<int> closed;
    for (int i = 0; i < n; ++i) {
        if (sizes[i] < 0) return PC_E_SCHEMA;
        const int u = union_ids[i];
        if (u < 0) continue;
        const bool continues = i > 0 && union_ids[i - 1] == u;
        if (!continues) {
            if (std::find(closed.begin(), closed.end(), u) != closed.end()) return PC_E_SCHEMA;
            closed.push_back(u);
        }
    }
    long next_free = 0;       // first position ID after everything laid out so far
    long union_start = 0;     // start shared by the children of the union being laid out
    for (int i = 0; i < n; ++i) {
        const int u = union_ids[i];
        const bool in_union = u >= 0;
        const bool continues = in_union && i > 0 && union_ids[i - 1] == u;
        if (!continues) union_start = next_free;
        const long begin = in_union ? union_start : next_free;
        starts[i] = (int)begin;
        next_free = std::max(next_free, begin + sizes[i]);
    }
    return next_free;
}

int pc_uncached_positions(int prev_start, int prev_len, int n_tokens, int32_t *pos)
{
    if (prev_start < 0 || prev_len < 0 || n_tokens < 0 || (n_tokens > 0 && !pos)) return PC_E_BADARG;
    const int first = prev_start + prev_len;
    for (int i = 0; i < n_tokens; ++i) pos[i] = first + i;
    return PC_OK;
}

int pc_check_selection(int n, const int *starts, const int *lens, int max_pos)
{
    return check_ranges(n, starts, lens, max_pos);
}

long pc_bytes_per_token(int n_layers, int n_kv_heads, int head_dim, int dtype)
{
    const int es = elem_size(dtype);
    if (n_layers <= 0 || n_kv_heads <= 0 || head_dim <= 0 || es == 0) return PC_E_BADARG;
    return (long)n_layers * 2 /* K and V */ * n_kv_heads * head_dim * es;
}

int pc_module_info(const pc_ctx *ctx, int layer, int module_id, int *n_tokens, int *start_pos)
{
    if (!ctx) return PC_E_BADARG;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return PC_E_LAYER;
    auto it = ctx->modules[layer].find(module_id);
    if (it == ctx->modules[layer].end()) return PC_E_UNKNOWN_MODULE;
    if (n_tokens) *n_tokens = it->second.n_tokens;
    if (start_pos) *start_pos = it->second.start_pos;
    return PC_OK;
}

int pc_pool_usage(const pc_ctx *ctx, size_t *used, size_t *total)
{
    if (!ctx) return PC_E_BADARG;
    if (used) *used = ctx->pool_used;
    if (total) *total = ctx->cfg.pool_bytes;
    return PC_OK;
}

int pc_last_attn_launch(const pc_ctx *ctx, int *n_splits, int *n_workgroups, int *waves_per_wg)
{
    if (!ctx) return PC_E_BADARG;
    if (n_splits) *n_splits = ctx->last_attn.n_splits;
    if (n_workgroups) *n_workgroups = ctx->last_attn.n_workgroups;
    if (waves_per_wg) *waves_per_wg = ctx->last_attn.waves_per_wg;
    return PC_OK;
}

}  // extern "C"
