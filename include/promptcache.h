/*
 * promptcache.h -- C ABI of the MI355X (gfx950) Prompt Cache hot path.
 *
 * The library implements the request-time part of Prompt Cache
 * (arXiv 2311.04934, Sec. 3.3 - 3.4 and Sec. 4.2):
 *
 *   1. prompt-module attention states (K, V), encoded once at the position IDs
 *      their schema fixes, are kept in a pool in HBM          (pc_store_module);
 *   2. a prompt that imports some of those modules gets its KV cache by
 *      concatenating the modules' states                      (pc_assemble_kv);
 *   3. the tokens of the prompt that are not cached are rotated at their own
 *      schema position IDs, their K/V are appended, and they attend over the
 *      assembled KV, which replaces the prefill               (pc_rope,
 *                                                 pc_append_kv, pc_prefill_attn).
 *
 * Conventions that hold for every call
 * ------------------------------------
 * Layout      Every K, V, Q and output tensor is token-major
 *             [tokens][heads][head_dim], head_dim contiguous, no padding.
 *             K/V tensors have n_kv_heads heads, Q/out have n_q_heads.
 *             Query head h reads KV head  h / (n_q_heads / n_kv_heads).
 * Element     pc_config.dtype: PC_F32 (4 bytes) or PC_BF16 (2 bytes, the upper
 *             half of an IEEE binary32, round-to-nearest-even on store).
 * Positions   int32 position IDs in [0, max_pos).  The assembled buffer is
 *             PACKED in the order modules are listed; a module left out of a
 *             prompt leaves a gap in the position IDs, never in the buffer.
 * RoPE        half-split pairing: element i rotates with element i + d/2 by the
 *             angle pos * rope_base^(-2i/d), i in [0, d/2).  Angles come from a
 *             table built in fp64 and indexed by position ID (Sec. 4.2).
 * Mask        key j is visible to query q  iff  pos[j] <= q_pos[q]: causality is
 *             decided by schema position IDs, not by buffer order.
 * "device"    pointer to GPU memory reachable from the current HIP device.
 * "host"      ordinary host memory; read (or written) before the call returns.
 * stream      a hipStream_t passed as void* (NULL = the default stream).  All
 *             device work is enqueued on it; no call synchronises or allocates
 *             device memory except pc_create / pc_destroy.
 * Ownership   The pool owns a copy of every stored module.  All other buffers
 *             belong to the caller and must stay valid until the stream has
 *             executed the call.
 * Errors      0 on success, a negative pc_status otherwise.  On error no device
 *             work has been enqueued by that call.  pc_strerror names the code.
 * Threads     a pc_ctx must not be used from two host threads at once.
 * Streams     attention calls of one context share its split-KV scratch: keep them
 *             on one stream (see pc_prefill_attn).  Assembly calls may run on another.
 */
#ifndef PROMPTCACHE_H
#define PROMPTCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pc_ctx pc_ctx;

typedef enum { PC_F32 = 0, PC_BF16 = 1 } pc_dtype;

typedef enum {
    PC_OK = 0,
    PC_E_BADARG = -1,         /* NULL pointer, negative size, misaligned buffer          */
    PC_E_LAYER = -2,          /* layer outside [0, n_layers)                             */
    PC_E_UNKNOWN_MODULE = -3, /* module id was never stored for that layer               */
    PC_E_OVERLAP = -4,        /* two selected modules share a position ID                */
    PC_E_CAPACITY = -5,       /* result does not fit the caller's buffer                 */
    PC_E_POOL_FULL = -6,      /* module pool exhausted                                   */
    PC_E_DUP_MODULE = -7,     /* id stored before with another length or start position  */
    PC_E_POS_RANGE = -8,      /* a position ID would fall outside [0, max_pos)           */
    PC_E_UNSUPPORTED = -9,    /* head_dim / dtype / head ratio the kernels do not cover  */
    PC_E_HIP = -10,           /* a HIP runtime call failed (no GPU, out of memory, ...)  */
    PC_E_SCHEMA = -11,        /* malformed schema description                            */
    PC_E_PARAM = -12          /* no such parameter, or argument longer than the parameter */
} pc_status;

typedef struct {
    int n_layers;
    int n_q_heads;
    int n_kv_heads;      /* must divide n_q_heads                                        */
    int head_dim;        /* PC_BF16: 64 or 128;  PC_F32: even, <= 256                    */
    int dtype;           /* pc_dtype                                                     */
    double rope_base;    /* e.g. 10000.0                                                 */
    int max_pos;         /* position IDs live in [0, max_pos)                            */
    size_t pool_bytes;   /* HBM reserved for stored modules, all layers together         */
    size_t scratch_bytes;/* HBM for split-KV partial results; 0 = library default        */
} pc_config;

/* ---------------------------------------------------------------- context */

/* Allocate the pool, the RoPE table (max_pos x head_dim/2 cos/sin pairs, computed
 * in fp64 on the host) and the split-KV scratch on the current HIP device. */
int pc_create(const pc_config *cfg, pc_ctx **out_ctx);

/* Synchronise the device and free everything pc_create allocated. */
int pc_destroy(pc_ctx *ctx);

const char *pc_strerror(int status);

/* ---------------------------------------------- the three calls of the path */

/*
 * Prompt-module encoding result -> pool  (Sec. 3.3; Sec. 4.1 "GPU memory").
 *
 * K, V       device, [n_tokens][n_kv_heads][head_dim].  K must already carry the
 *            positional encoding for positions start_pos .. start_pos+n_tokens-1
 *            (that is what the model emits when the module is encoded at its
 *            schema positions); V is position-free.  Both are copied
 *            (device-to-device, asynchronously on `stream`).
 * module_id  any non-negative int, unique per layer.  Storing an id again with
 *            the same n_tokens and start_pos overwrites its states (modules may
 *            be refreshed at run time); with different ones: PC_E_DUP_MODULE.
 * Errors     PC_E_LAYER, PC_E_BADARG, PC_E_POS_RANGE, PC_E_POOL_FULL,
 *            PC_E_DUP_MODULE.
 */
int pc_store_module(pc_ctx *ctx, int layer, int module_id, const void *K, const void *V,
                    int n_tokens, int start_pos, void *stream);

/*
 * Cached inference, step 1: concatenate the imported modules' states (Sec. 3.4,
 * "(k_C, v_C) = (concat(k_A, k_B), concat(v_A, v_B))").  One bandwidth-bound
 * gather kernel; bytes are copied verbatim.
 *
 * module_ids      host, n_modules ids, in the order they are to appear in the
 *                 buffer (any order is valid: the mask works on positions).
 * out_K, out_V    device, caller-owned, room for capacity_tokens rows of
 *                 n_kv_heads*head_dim elements, 16-byte aligned.
 *                 Row r of module m lands at row (sum of lengths of the modules
 *                 listed before m) + r.
 * out_pos         device, int32[capacity_tokens]; row r of module m gets
 *                 start_pos(m) + r.
 * out_n_tokens    host, receives the number of rows written (may be NULL).
 * Errors          PC_E_UNKNOWN_MODULE (an import the pool does not hold),
 *                 PC_E_OVERLAP (e.g. two children of one union), PC_E_CAPACITY,
 *                 PC_E_LAYER, PC_E_BADARG.
 */
int pc_assemble_kv(pc_ctx *ctx, int layer, const int *module_ids, int n_modules,
                   void *out_K, void *out_V, int32_t *out_pos, int capacity_tokens,
                   int *out_n_tokens, void *stream);

/*
 * Cached inference, step 2: attention of the uncached tokens over the assembled
 * KV, which stands in for the prefill (Sec. 3.4, "using (k_C, v_C) as a KV cache").
 *
 *   out[q][h] = sum_j softmax_j( rope(Q_new[q][h], q_pos[q]) . asm_K[j][kv(h)] / sqrt(d) )
 *               * asm_V[j][kv(h)]        over rows j with asm_pos[j] <= q_pos[q].
 *
 * Q_new    device, [n_q][n_q_heads][head_dim], NOT yet rotated: the rotation at
 *          q_pos is fused into this call.  Not modified.
 * q_pos    device, int32[n_q] schema position IDs of the uncached tokens.
 * asm_K/V  device, [n_kv][n_kv_heads][head_dim]: the assembled modules, normally
 *          followed by the uncached tokens' own K/V (pc_append_kv).
 * asm_pos  device, int32[n_kv].
 * out      device, [n_q][n_q_heads][head_dim] in the context dtype.  A query with
 *          no visible key gets zeros.
 * PC_BF16: QK^T and PV run on bf16 MFMA with fp32 accumulation and fp32 softmax
 * statistics; PC_F32: everything in fp32.  The work is split over the KV axis
 * when that is needed to fill the GPU; partial results go through the context's
 * scratch and a small merge kernel, all on `stream`.  A scratch too small for the
 * wanted number of splits is no error: the call then runs with as many splits as
 * fit (down to one, which needs none).
 * The context has ONE scratch: attention calls of one context (every
 * pc_prefill_attn* call) must be enqueued on one stream, or be ordered by the
 * caller; two of them running at once would overwrite each other's partials.
 * Errors   PC_E_LAYER, PC_E_BADARG.
 */
int pc_prefill_attn(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos, int n_q,
                    const void *asm_K, const void *asm_V, const int32_t *asm_pos, int n_kv,
                    void *out, void *stream);

/*
 * pc_prefill_attn for callers that cannot allocate device memory or hand the library any:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same result (bit for bit: the same launch decomposition).  The split-KV partials go to
 * a fixed array of PC_STATIC_SCRATCH_BYTES that is part of the library's device code (one copy per
 * GPU, held until the process ends) instead of the context's scratch; the call allocates nothing
 * and clears nothing (every byte it reads it has written in the same call).
 * A launch whose partials exceed the array is refused with PC_E_CAPACITY and nothing is enqueued
 * (partials take n_splits * n_q * n_q_heads * (2 * head_dim + 8) bytes, about 17 MB when one split
 * pass fills the GPU and at most twice that).
 * All calls on one GPU share that GPU's array, whichever context or stream they use: two
 * pc_prefill_attn_static calls that overlap in time on one GPU race.  Order them on one stream.
 */
#define PC_STATIC_SCRATCH_BYTES (32u << 20)
int pc_prefill_attn_static(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos, int n_q,
                           const void *asm_K, const void *asm_V, const int32_t *asm_pos, int n_kv,
                           void *out, void *stream);

/* --------------------------------------------------------- supporting calls */

/*
 * RoPE at arbitrary position IDs, in place (Sec. 3.3: module positions do not
 * start at zero; Sec. 4.2: rotation looked up by position ID).
 * x device [n_tokens][n_heads][head_dim]; pos device int32[n_tokens], every
 * value in [0, max_pos) (the caller guarantees it; the kernel clamps).
 */
int pc_rope(pc_ctx *ctx, void *x, int n_tokens, int n_heads, const int32_t *pos, void *stream);

/*
 * Append the uncached tokens' own states behind the assembled modules
 * (Sec. 3.4: the new segments' states are concatenated with the cached ones to
 * give the states of the entire prompt).
 * K_new_raw  device [n_q][n_kv_heads][head_dim], not rotated; rotated at q_pos on
 *            the way.   V_new  device, same shape, copied.
 * Rows n_kv_before .. n_kv_before+n_q-1 of asm_K/asm_V/asm_pos are written.
 * Errors     PC_E_CAPACITY if n_kv_before + n_q > capacity_tokens.
 */
int pc_append_kv(pc_ctx *ctx, int layer, const void *K_new_raw, const void *V_new,
                 const int32_t *q_pos, int n_q, void *asm_K, void *asm_V, int32_t *asm_pos,
                 int n_kv_before, int capacity_tokens, void *stream);

/* ------------------------------------------- batched (several prompts at once) */

/* Position ID of an assembled row that holds no token (an unused placeholder of a
 * parameter): larger than any query position, so no query ever sees the row. */
#define PC_POS_NONE 0x7fffffff

/*
 * Sec. 3.2.2 "Maximizing reuse with parameters", Sec. 3.3 (last paragraph): a module may
 * contain parameters, runs of `len` placeholder tokens whose position IDs are fixed at
 * encoding time.  pc_set_module_params records, for module_id in every layer, that rows
 * [offsets[j], offsets[j]+lens[j]) of the module are parameter j (host arrays; ranges
 * sorted, disjoint, non-negative; n_params = 0 clears).  It replaces an earlier record.
 * Errors: PC_E_BADARG.
 */
int pc_set_module_params(pc_ctx *ctx, int module_id, int n_params, const int *offsets, const int *lens);

/*
 * Supply arguments to parameters of the modules of an assembled prompt (same section).
 * module_ids/n_modules is the list that pc_assemble_kv was called with (it fixes where each
 * module's rows are).  Argument a belongs to parameter arg_param[a] of module
 * module_ids[arg_module[a]] and consists of rows arg_offsets[a] .. arg_offsets[a+1]-1 of
 * K_arg_raw / V_arg (device, [tokens][n_kv_heads][head_dim], keys not yet rotated).  Its
 * tokens take the placeholders' position IDs in order; the rotated keys and the values
 * overwrite the placeholders' rows of asm_K / asm_V.  An argument may be shorter than the
 * parameter: the remaining placeholder rows keep their states but get position PC_POS_NONE,
 * so they are tokens no more.  A parameter that gets no argument is left as encoded.
 * One kernel launch on `stream`; host arrays: module_ids, arg_module, arg_param,
 * arg_offsets (int[n_args+1]).  Errors: PC_E_LAYER, PC_E_UNKNOWN_MODULE, PC_E_BADARG,
 * PC_E_PARAM (unknown parameter, range outside the module, argument too long),
 * PC_E_CAPACITY (the modules do not fit capacity_tokens); nothing is enqueued on error.
 */
int pc_fill_params(pc_ctx *ctx, int layer, const int *module_ids, int n_modules, int n_args,
                   const int *arg_module, const int *arg_param, const int *arg_offsets,
                   const void *K_arg_raw, const void *V_arg, void *asm_K, void *asm_V,
                   int32_t *asm_pos, int capacity_tokens, void *stream);

/*
 * Sec. 3.4 "batch inference": B prompts derived from one schema, possibly
 * importing the same module.  Buffers are packed: prompt b owns rows
 * kv_offsets[b] .. kv_offsets[b+1]-1 of out_K/out_V/out_pos (that span is its
 * capacity, sized by the caller to also hold the tokens appended later) and its
 * modules fill the first out_n_tokens[b] of them.  A shared module is read from
 * the pool once per prompt that imports it (copying form of batch sharing).
 *
 * module_ids_flat  host, ids of prompt 0, then prompt 1, ...
 * mod_offsets      host int[B+1]: prompt b imports module_ids_flat[mod_offsets[b] .. mod_offsets[b+1])
 * kv_offsets       host int[B+1], non-decreasing row offsets
 * out_n_tokens     host int[B]
 */
int pc_assemble_kv_batched(pc_ctx *ctx, int layer, const int *module_ids_flat, const int *mod_offsets,
                           int n_prompts, void *out_K, void *out_V, int32_t *out_pos,
                           const int *kv_offsets, int *out_n_tokens, void *stream);

/*
 * Sec. 3.4: bringing the cached modules in is a copy of stored states and does not depend on the
 * forward pass, so the modules of ALL layers can be concatenated when the request arrives, before
 * the first layer runs.  This call does pc_assemble_kv_batched for layers first_layer ..
 * first_layer+n_layers-1 with as few kernel launches as the kernels' segment tables allow (64
 * module segments and 32 layers per launch), which spreads a launch's fixed cost over gigabytes
 * instead of tens of megabytes.  The uncached tokens' rows are appended per layer afterwards
 * (pc_append_kv_batched / pc_append_rotate_batched), when the forward pass has produced them.
 *
 * out_K, out_V, out_pos   HOST arrays of n_layers device pointers: layer first_layer+l is assembled
 *                         into out_K[l], out_V[l], out_pos[l], each laid out like the buffers of
 *                         pc_assemble_kv_batched (same kv_offsets for every layer), 16-byte aligned.
 * The other arguments, the result per layer and the errors are those of pc_assemble_kv_batched;
 * PC_E_LAYER if the layer range leaves [0, n_layers).  Every layer is validated before the first
 * launch: on error nothing has been enqueued.
 */
int pc_assemble_kv_layers(pc_ctx *ctx, int first_layer, int n_layers, const int *module_ids_flat,
                          const int *mod_offsets, int n_prompts, void *const *out_K, void *const *out_V,
                          int32_t *const *out_pos, const int *kv_offsets, int *out_n_tokens,
                          void *stream);

/* Batched pc_append_kv.  Prompt b's new tokens are rows q_offsets[b] .. q_offsets[b+1]-1
 * of K_new_raw/V_new/q_pos and go to rows kv_offsets[b]+kv_lens[b] ... of the packed
 * buffer; they must fit below kv_offsets[b+1].  All offset arrays are host. */
int pc_append_kv_batched(pc_ctx *ctx, int layer, const void *K_new_raw, const void *V_new,
                         const int32_t *q_pos, const int *q_offsets, int n_prompts, void *asm_K,
                         void *asm_V, int32_t *asm_pos, const int *kv_offsets, const int *kv_lens,
                         void *stream);

/*
 * Sec. 3.4: a prompt's KV cache is its imported modules followed by its own uncached
 * tokens.  This call does pc_assemble_kv_batched and pc_append_kv_batched (with kv_lens =
 * the assembled row counts) in ONE kernel launch: the two steps write disjoint rows of the
 * same packed buffers, and the append alone is cheaper than a launch.  Arguments as in the
 * two calls; out_n_tokens[b] (host) receives prompt b's total rows, modules plus new
 * tokens.  PC_E_CAPACITY if a prompt's span kv_offsets[b+1]-kv_offsets[b] cannot hold both.
 * Falls back to two launches when the batch has more than 64 module segments or prompts.
 */
int pc_assemble_append_kv_batched(pc_ctx *ctx, int layer, const int *module_ids_flat,
                                  const int *mod_offsets, int n_prompts, const void *K_new_raw,
                                  const void *V_new, const int32_t *q_pos, const int *q_offsets,
                                  void *out_K, void *out_V, int32_t *out_pos, const int *kv_offsets,
                                  int *out_n_tokens, void *stream);

/* Batched pc_prefill_attn.  Prompt b's queries are rows q_offsets[b] .. q_offsets[b+1]-1
 * of Q_new/q_pos/out and see rows kv_offsets[b] .. kv_offsets[b]+kv_lens[b]-1 of the
 * packed KV.  q_offsets host int[B+1]; kv_offsets host int[B+1]; kv_lens host int[B]. */
int pc_prefill_attn_batched(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos,
                            const int *q_offsets, int n_prompts, const void *asm_K, const void *asm_V,
                            const int32_t *asm_pos, const int *kv_offsets, const int *kv_lens,
                            void *out, void *stream);

/*
 * Sec. 4.2 (rotation looked up by position ID), applied once per token instead of once per
 * attention workgroup: the calls below do what pc_append_kv_batched /
 * pc_assemble_append_kv_batched do and, in the same launch, also write
 *     Q_rot[row] = rotation of Q_new[row] at q_pos[row], times the attention kernels' score scale
 * (Q_new, Q_rot: device [total_q, n_q_heads, head_dim], 16-byte aligned, distinct buffers; under
 * pc_set_alibi the rows are only scaled).  Q_rot is an operand for the *_rotated attention calls
 * and nothing else: the scale folded in is 1/sqrt(head_dim) for fp32 contexts and
 * log2(e)/sqrt(head_dim) for bf16 ones.
 *   pc_append_rotate_batched            arguments of pc_append_kv_batched + Q_new, Q_rot
 *   pc_assemble_append_rotate_batched   arguments of pc_assemble_append_kv_batched + Q_new, Q_rot
 *   pc_prefill_attn_rotated_batched,
 *   pc_prefill_attn_shared_rotated_batched   as their namesakes, with Q_rot in place of Q_new; the
 *                                        results are those of the namesakes on Q_new
 * Every attention workgroup otherwise rotates its queries itself, once per KV split; with the
 * rotation done here that part of the kernels' prologue goes away.
 */
int pc_append_rotate_batched(pc_ctx *ctx, int layer, const void *K_new_raw, const void *V_new,
                             const void *Q_new, const int32_t *q_pos, const int *q_offsets,
                             int n_prompts, void *asm_K, void *asm_V, int32_t *asm_pos,
                             const int *kv_offsets, const int *kv_lens, void *Q_rot, void *stream);
int pc_assemble_append_rotate_batched(pc_ctx *ctx, int layer, const int *module_ids_flat,
                                      const int *mod_offsets, int n_prompts, const void *K_new_raw,
                                      const void *V_new, const void *Q_new, const int32_t *q_pos,
                                      const int *q_offsets, void *out_K, void *out_V, int32_t *out_pos,
                                      const int *kv_offsets, int *out_n_tokens, void *Q_rot,
                                      void *stream);
int pc_prefill_attn_rotated_batched(pc_ctx *ctx, int layer, const void *Q_rot, const int32_t *q_pos,
                                    const int *q_offsets, int n_prompts, const void *asm_K,
                                    const void *asm_V, const int32_t *asm_pos, const int *kv_offsets,
                                    const int *kv_lens, void *out, void *stream);
int pc_prefill_attn_shared_rotated_batched(pc_ctx *ctx, int layer, const void *Q_rot,
                                           const int32_t *q_pos, const int *q_offsets, int n_prompts,
                                           const int *module_ids_flat, const int *mod_offsets,
                                           const void *K_tail, const void *V_tail, void *out,
                                           void *stream);

/*
 * Sec. 3.3 ("attention masking effect"), scaffolding: a scaffold is a set of prompt modules
 * that was ALSO encoded jointly, so that its members share one attention span.  When a prompt
 * imports every member of a scaffold, the jointly encoded states override the members' own.
 * To this library the joint encoding is one more stored module per member: override_ids[i]
 * names the states (stored with pc_store_module / pc_store_module_host, same length and first
 * position ID as member_ids[i]) that stand in for member_ids[i].
 *
 * pc_define_scaffold     registers one scaffold (host int arrays of n_members ids, members
 *                        distinct).  From then on every call that takes import lists
 *                        (pc_assemble_kv*, pc_assemble_append_kv_batched,
 *                        pc_prefill_attn_shared_batched) applies the rule per prompt: scaffolds
 *                        in definition order; one that would touch a member an earlier scaffold
 *                        has overridden is skipped.  An override id that was never stored for the
 *                        layer gives PC_E_UNKNOWN_MODULE at that call, one whose length or first
 *                        position differs from its member's PC_E_SCHEMA.
 * pc_resolve_scaffolds   the rule itself on host integers, no context: scaffold s has members
 *                        member_ids[scaffold_offsets[s] .. scaffold_offsets[s+1]-1] and the
 *                        override ids at the same indices; out_ids[n_ids] receives the import list
 *                        with the overridden ids replaced where they stood.
 */
int pc_define_scaffold(pc_ctx *ctx, int n_members, const int *member_ids, const int *override_ids);
int pc_resolve_scaffolds(int n_ids, const int *ids, int n_scaffolds, const int *scaffold_offsets,
                         const int *member_ids, const int *override_ids, int *out_ids);

/*
 * Sec. 4.2, ALiBi: models that encode position as a linear bias on the attention scores
 * instead of a rotation.  The bias follows the given position IDs:
 *     score(q, k) = Q.K / sqrt(d)  -  slope[head] * (pos_q - pos_k),   visible iff pos_k <= pos_q.
 *
 * pc_set_alibi     slopes: HOST float[n_q_heads], finite and >= 0 (PC_E_BADARG otherwise); the
 *                  context switches to the linear bias: pc_prefill_attn* add it and use Q as it
 *                  is, pc_append_kv*, pc_assemble_append_kv_batched and pc_fill_params store keys
 *                  unrotated (modules must then be stored unrotated too).  slopes == NULL switches
 *                  back to rotation.  A set-up call: it copies synchronously and must not overlap
 *                  with attention calls in flight on the context.
 *                  Every dtype and head_dim the rotary path serves.
 * pc_alibi_slopes  the sequence that encoding's authors define (host helper, no context):
 *                  n a power of two: 2^(-8/n), 2^(-16/n), ...; otherwise the sequence of the
 *                  largest power of two below n followed by the odd members of the next one.
 */
int pc_set_alibi(pc_ctx *ctx, const float *slopes);
int pc_alibi_slopes(int n_heads, float *slopes);

/*
 * Sec. 4.1: prompt modules kept in CPU memory (capacity of host DRAM instead of HBM, at the
 * price of a host-to-device copy at every use; Sec. 5.4 measures that copy).
 *
 * pc_host_pool_reserve    allocates the context's host pool once: `bytes` of pinned host memory
 *                         that the GPU can address.  PC_E_BADARG if a pool exists already or
 *                         bytes == 0, PC_E_HIP if the allocation fails.
 * pc_store_module_host    like pc_store_module, but K_host/V_host are HOST pointers
 *                         ([n_tokens, n_kv_heads, head_dim], position-encoded keys) and the copy
 *                         into the host pool is done by the CPU before the call returns; the
 *                         caller keeps ownership of its buffers.  A module lives in the tier it
 *                         was first stored in: storing an id again in the other tier is
 *                         PC_E_DUP_MODULE.  Refreshing a host module while an assembly that reads
 *                         it is still running on the GPU is a race the caller must avoid.
 *                         PC_E_POOL_FULL if no host pool was reserved or it cannot hold the module.
 * pc_set_host_copy_mode   how the assemble calls (pc_assemble_kv, pc_assemble_kv_batched,
 *                         pc_assemble_append_kv_batched) bring host-resident modules in:
 *                         PC_HOST_READ_KERNEL (default): the assembly kernel loads them from the
 *                         pinned pool over the host link, in the same single launch as the
 *                         HBM-resident modules; PC_HOST_COPY_ENGINE: one hipMemcpyAsync per module
 *                         and tensor on the caller's stream straight into the packed buffer, the
 *                         kernel then writes only those rows' position IDs.
 * All other calls take module ids of either tier, except pc_prefill_attn_shared_batched, which
 * refuses host-resident modules (PC_E_UNSUPPORTED): they have to be assembled first.
 * The result of an assembly is bit-identical whichever tier and mode served it.
 */
#define PC_HOST_READ_KERNEL 0
#define PC_HOST_COPY_ENGINE 1
int pc_host_pool_reserve(pc_ctx *ctx, size_t bytes);
int pc_store_module_host(pc_ctx *ctx, int layer, int module_id, const void *K_host, const void *V_host,
                         int n_tokens, int start_pos);
int pc_set_host_copy_mode(pc_ctx *ctx, int mode);

/*
 * Sec. 3.4 (sharing modules between the prompts of a batch instead of copying them) and
 * Sec. 3.3: attention of every prompt's uncached tokens over its imported modules READ IN
 * PLACE from the module pool, followed by the uncached tokens' own rows.  No packed KV
 * buffer is assembled; a module imported by many prompts is read from its one copy.
 * The result equals pc_assemble_append_kv_batched + pc_prefill_attn_batched.
 *   module_ids_flat, mod_offsets  host, as in pc_assemble_kv_batched: prompt b imports
 *                       module_ids_flat[mod_offsets[b] .. mod_offsets[b+1]-1], in this order;
 *                       their position ranges must not overlap (PC_E_OVERLAP).
 *   Q_new, q_pos, q_offsets, out  as in pc_prefill_attn_batched.
 *   K_tail, V_tail      device [total_q, n_kv_heads, head_dim], 16-byte aligned: the uncached
 *                       tokens' keys ALREADY ROTATED to q_pos, and values, row q_offsets[b]+i
 *                       for prompt b's token i (what pc_append_kv_batched writes into an
 *                       empty buffer with kv_offsets = q_offsets and kv_lens = 0).
 * Every dtype and head_dim the packed path serves; at most 63 modules per prompt
 * (PC_E_UNSUPPORTED beyond).  Inputs are read, never written; ownership stays with the caller.
 */
int pc_prefill_attn_shared_batched(pc_ctx *ctx, int layer, const void *Q_new, const int32_t *q_pos,
                                   const int *q_offsets, int n_prompts, const int *module_ids_flat,
                                   const int *mod_offsets, const void *K_tail, const void *V_tail,
                                   void *out, void *stream);

/* ----------------------------------------------- host-side integer helpers */

/*
 * Schema position layout (Sec. 3.3): an entry starts where the entries before
 * it end (predecessors of 50 and 60 tokens -> start 110); the children of a
 * union share one start and the union spans its largest child (Sec. 3.2.3).
 * sizes, union_ids, starts: host int[n]; union_ids[i] < 0 for an ordinary module,
 * otherwise the id of its union, whose children must be adjacent.
 * Returns the schema's total span (>= 0) or PC_E_SCHEMA.
 */
long pc_schema_layout(int n, const int *sizes, const int *union_ids, int *starts);

/* Position IDs of a run of uncached text that follows an imported module
 * (Sec. 3.4): prev_start + prev_len + i.  Text at the very start of a prompt uses
 * prev_start = prev_len = 0.  pos: host int32[n_tokens]. */
int pc_uncached_positions(int prev_start, int prev_len, int n_tokens, int32_t *pos);

/* Would these modules be accepted together?  PC_OK, PC_E_OVERLAP, PC_E_POS_RANGE or
 * PC_E_BADARG.  starts, lens: host int[n]. */
int pc_check_selection(int n, const int *starts, const int *lens, int max_pos);

/* K+V bytes one cached token occupies over all layers (the closed form behind
 * Table 2, with n_kv_heads*head_dim in place of the hidden size). */
long pc_bytes_per_token(int n_layers, int n_kv_heads, int head_dim, int dtype);

/* Look a stored module up: PC_OK and its length/start, or PC_E_UNKNOWN_MODULE. */
int pc_module_info(const pc_ctx *ctx, int layer, int module_id, int *n_tokens, int *start_pos);

/*
 * Calibration for benchmarks (synchronous, allocate and free their own buffers; not for the
 * request path): what this machine sustains on the two roofs the kernels are held against.
 *   pc_calib_copy   a plain device-to-device copy kernel over `bytes` bytes, `repeats` launches;
 *                   *gb_per_s = read + written bytes per second.
 *   pc_calib_mfma   one workgroup of 8 waves per CU, each wave issuing iters x 16
 *                   v_mfma_f32_32x32x16_bf16 on independent accumulators and nothing else;
 *                   *tflop_per_s = dense bf16 rate reached.
 */
int pc_calib_copy(pc_ctx *ctx, size_t bytes, int repeats, double *gb_per_s);
int pc_calib_mfma(pc_ctx *ctx, int iters, double *tflop_per_s);

/*
 * Sec. 3.4 (a prompt's imports are validated and its modules retrieved once): every call that takes
 * import lists keeps the validated plan of its last few distinct lists, so the same lists at the next
 * layer or the next step cost an integer comparison: no look-up, no sort, no host allocation.
 * Storing a new module or defining a scaffold discards the kept plans.
 * pc_plan_stats (for tests and benchmarks): calls served from a kept plan, calls that had to plan, and
 * the number of host heap allocations the planning code has made so far on the calling thread.
 */
int pc_plan_stats(const pc_ctx *ctx, long *hits, long *misses, long *heap_allocs);

/* Bytes of pool in use / total. */
int pc_pool_usage(const pc_ctx *ctx, size_t *used, size_t *total);

/*
 * Which bf16 attention kernel serves head_dim 128.  PC_ATTN_AUTO (default): the kernel that stages
 * K/V with asynchronous global->LDS copies, which addresses a prompt's packed K (or V) with 32-bit
 * offsets, and the register-staged kernel (64-bit offsets) for prompts whose packed K exceeds 4 GiB.
 * PC_ATTN_REGISTER_STAGED: the register-staged kernel for every packed-buffer call (tests and
 * comparisons; calls that read modules in place keep the automatic choice).  No effect on
 * head_dim 64 and fp32, which have one kernel each.
 */
#define PC_ATTN_AUTO 0
#define PC_ATTN_REGISTER_STAGED 1
int pc_set_attn_kernel(pc_ctx *ctx, int which);

/* How the last pc_prefill_attn[_batched] call was launched: number of KV splits,
 * workgroups of the main kernel and waves per workgroup (for benchmarks). */
int pc_last_attn_launch(const pc_ctx *ctx, int *n_splits, int *n_workgroups, int *waves_per_wg);

/*
 * Optional per-kernel timing for benchmarks.  pc_profile_enable(ctx, n) creates n HIP event
 * pairs per kernel kind (n = 0 turns profiling off and frees them; it synchronises the
 * device).  While enabled, every kernel the library launches carries one pair of its kind
 * (until they are used up), which then holds that kernel's own begin and end timestamps on
 * the stream it ran on.  pc_profile_read waits for the recorded events of one kind, returns
 * how many launches were timed and the sum of their durations in milliseconds, and resets
 * that kind's counter.  pc_profile_read_each does the same and also copies the first
 * `capacity` durations (milliseconds, launch order) to the host array ms_out.
 * kind: 0 gather (pc_assemble_kv*, pc_assemble_append_kv_batched), 1 append, 2 attention
 * main kernel, 3 split-KV merge, 4 pc_rope.
 */
int pc_profile_enable(pc_ctx *ctx, int max_records_per_kind);
int pc_profile_read(pc_ctx *ctx, int kind, int *n_records, double *total_ms);
int pc_profile_read_each(pc_ctx *ctx, int kind, float *ms_out, int capacity, int *n_records,
                         double *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* PROMPTCACHE_H */
