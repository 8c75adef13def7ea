/*
 * pc_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 CPU statement of what the Prompt Cache hot path computes,
 * written from the paper (arXiv 2311.04934).  It exists so that the GPU library
 * can be checked against something that shares no code with it.  Only tests,
 * the smoke check and the benchmark's "cpu_baseline" leg may call it; the
 * product path never does.
 *
 * Every function is the textbook definition written out as loops: no blocking,
 * no fusion, no online softmax, no tables.  The only concession to speed is an
 * optional OpenMP "parallel for" over independent (query, head) pairs, which
 * does not change any arithmetic or its order inside a pair.
 *
 * Conventions (shared with the GPU library only through the C header's prose):
 *   tensors are token-major  [tokens][heads][d],  d contiguous;
 *   position IDs are int32;
 *   RoPE pairs element i with element i + d/2 (half-split pairing) and uses
 *   theta_i = base^(-2i/d);
 *   a key is visible to a query iff  pos_k <= pos_q.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* threads                                                             */
/* ------------------------------------------------------------------ */

static int g_threads = 1;

/* Set the number of OpenMP threads the attention loops use; returns the
 * number actually in effect (1 when built without OpenMP). */
int orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n < 1) n = 1;
    g_threads = n;
    return g_threads;
#else
    (void)n;
    g_threads = 1;
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Schema layout  (Sec. 3.3 "Encoding schema", Sec. 3.2.3 union rule)   */
/* ------------------------------------------------------------------ */

/*
 * Start position of every schema entry.
 *
 * A module's first position ID is its absolute location in the schema: the
 * sum of the sizes of everything before it (two predecessors of 50 and 60
 * tokens put the next module at 110).  Children of one union all start at the
 * same position, and the union as a whole occupies as many positions as its
 * largest child.
 *
 * size[i]      token count of entry i (schema order)
 * union_id[i]  < 0: ordinary module; >= 0: child of that union.  Children of
 *              one union must be adjacent in schema order.
 * start[i]     (out) first position ID of entry i
 * returns      total number of position IDs the schema spans, or -1 when a
 *              union's children are not adjacent or a size is negative.
 */
long orc_layout(int n, const int *size, const int *union_id, int *start)
{
    long cursor = 0;
    int i = 0;
    /* a union id may not reappear once its run has ended */
    for (int a = 0; a < n; ++a) {
        if (size[a] < 0) return -1;
        if (union_id[a] < 0) continue;
        for (int b = a + 1; b < n; ++b)
            if (union_id[b] == union_id[a])
                for (int c = a + 1; c < b; ++c)
                    if (union_id[c] != union_id[a]) return -1;
    }
    while (i < n) {
        if (union_id[i] < 0) {
            start[i] = (int)cursor;
            cursor += size[i];
            ++i;
        } else {
            int u = union_id[i];
            int widest = 0;
            int j = i;
            while (j < n && union_id[j] == u) {
                start[j] = (int)cursor;
                if (size[j] > widest) widest = size[j];
                ++j;
            }
            cursor += widest;
            i = j;
        }
    }
    return cursor;
}

/*
 * Position IDs of a run of uncached text (Sec. 3.4): text that follows an
 * imported module continues from that module's last position + 1; text at the
 * very beginning of the prompt starts at 0.
 *
 * prev_start/prev_len  the imported module the text comes after
 *                      (prev_len == 0 and prev_start == 0: start of prompt)
 */
void orc_text_positions(int prev_start, int prev_len, int n_tokens, int32_t *pos)
{
    for (int i = 0; i < n_tokens; ++i) pos[i] = prev_start + prev_len + i;
}

/* ------------------------------------------------------------------ */
/* RoPE at arbitrary position IDs  (Sec. 3.3, Sec. 4.2)                 */
/* ------------------------------------------------------------------ */

/*
 * In-place rotary embedding of x[n_tokens][n_heads][d] at the given position
 * IDs.  For each pair (x[i], x[i + d/2]), i in [0, d/2):
 *     angle = pos * base^(-2i/d)
 *     x[i]       <- x[i] cos(angle) - x[i+d/2] sin(angle)
 *     x[i+d/2]   <- x[i+d/2] cos(angle) + x[i] sin(angle)
 * The paper only requires that the rotation be looked up by position ID, so
 * any integer position (not only 0..n-1) is accepted.
 */
void orc_rope(double *x, int n_tokens, int n_heads, int d, const int32_t *pos, double base)
{
    int half = d / 2;
    for (int t = 0; t < n_tokens; ++t) {
        for (int h = 0; h < n_heads; ++h) {
            double *v = x + ((size_t)t * n_heads + h) * d;
            for (int i = 0; i < half; ++i) {
                double theta = pow(base, -2.0 * (double)i / (double)d);
                double angle = (double)pos[t] * theta;
                double c = cos(angle), s = sin(angle);
                double lo = v[i], hi = v[i + half];
                v[i] = lo * c - hi * s;
                v[i + half] = hi * c + lo * s;
            }
        }
    }
}

/* ------------------------------------------------------------------ */
/* KV assembly  (Sec. 3.4: "concatenating the KV state tensors")        */
/* ------------------------------------------------------------------ */

/*
 * Concatenate the selected modules' K and V rows, in the order given, into a
 * packed buffer, and write each row's schema position ID.  Pure byte copy:
 * the states are opaque here.  Gaps left by omitted modules show up only in
 * out_pos, never as holes in the buffer.
 *
 * mod_K[m], mod_V[m]  bytes of selected module m, mod_len[m] rows of row_bytes
 * mod_start[m]        its first schema position ID
 * returns             number of rows written
 */
long orc_assemble(int n_sel, const uint8_t *const *mod_K, const uint8_t *const *mod_V,
                  const int *mod_len, const int *mod_start, size_t row_bytes,
                  uint8_t *out_K, uint8_t *out_V, int32_t *out_pos)
{
    long row = 0;
    for (int m = 0; m < n_sel; ++m) {
        for (int i = 0; i < mod_len[m]; ++i) {
            for (size_t b = 0; b < row_bytes; ++b) {
                out_K[(size_t)row * row_bytes + b] = mod_K[m][(size_t)i * row_bytes + b];
                out_V[(size_t)row * row_bytes + b] = mod_V[m][(size_t)i * row_bytes + b];
            }
            out_pos[row] = mod_start[m] + i;
            ++row;
        }
    }
    return row;
}

/* ------------------------------------------------------------------ */
/* Attention of uncached tokens over the assembled KV  (Sec. 3.4)       */
/* ------------------------------------------------------------------ */

/* softmax(s) . V for one (query row, head); s already holds -inf where masked */
static void softmax_times_v(const double *s, int n, const double *V, int v_stride, int d, double *out)
{
    double top = -INFINITY;
    for (int j = 0; j < n; ++j)
        if (s[j] > top) top = s[j];
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    if (top == -INFINITY) return; /* no visible key: defined as zeros */
    double denom = 0.0;
    for (int j = 0; j < n; ++j)
        if (s[j] != -INFINITY) denom += exp(s[j] - top);
    for (int j = 0; j < n; ++j) {
        if (s[j] == -INFINITY) continue;
        double p = exp(s[j] - top) / denom;
        const double *v = V + (size_t)j * v_stride;
        for (int c = 0; c < d; ++c) out[c] += p * v[c];
    }
}

/*
 * out[q][h][:] = sum_j softmax_j( rope(Q[q][h], q_pos[q]) . K[j][kv(h)] / sqrt(d) ) V[j][kv(h)]
 * over the keys j with k_pos[j] <= q_pos[q];  kv(h) = h / (Hq / Hkv).
 *
 * Q is raw (not yet rotated): the rotation at q_pos is part of this step.
 * K is already position-encoded (that is what a prompt module stores) and V
 * is position-free.  This is exactly "run the uncached tokens through
 * attention using the concatenated module states as the KV cache", with the
 * causal rule stated on position IDs so that it does not depend on the order
 * in which modules were concatenated.
 *
 * Q   [nq][Hq][d]    K,V [nkv][Hkv][d]    out [nq][Hq][d]
 */
void orc_attn(const double *Q, const int32_t *q_pos, int nq, const double *K, const double *V,
              const int32_t *k_pos, int nkv, int Hq, int Hkv, int d, double base, double *out)
{
    int group = Hq / Hkv;
    double inv_sqrt_d = 1.0 / sqrt((double)d);
    long pairs = (long)nq * Hq;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 4) num_threads(g_threads)
#endif
    for (long w = 0; w < pairs; ++w) {
        int q = (int)(w / Hq), h = (int)(w % Hq);
        int kvh = h / group;
        double *qrot = (double *)malloc(sizeof(double) * (size_t)d);
        double *s = (double *)malloc(sizeof(double) * (size_t)(nkv > 0 ? nkv : 1));
        memcpy(qrot, Q + ((size_t)q * Hq + h) * d, sizeof(double) * (size_t)d);
        orc_rope(qrot, 1, 1, d, q_pos + q, base);
        for (int j = 0; j < nkv; ++j) {
            if (k_pos[j] <= q_pos[q]) {
                const double *k = K + ((size_t)j * Hkv + kvh) * d;
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += qrot[c] * k[c];
                s[j] = dot * inv_sqrt_d;
            } else {
                s[j] = -INFINITY;
            }
        }
        softmax_times_v(s, nkv, V + (size_t)kvh * d, Hkv * d, d, out + ((size_t)q * Hq + h) * d);
        free(s);
        free(qrot);
    }
}

/* ------------------------------------------------------------------ */
/* ALiBi at arbitrary position IDs  (Sec. 4.2, "ALiBi")                 */
/* ------------------------------------------------------------------ */

/*
 * Per-head slopes of the linear attention bias as its authors define them:
 * for a power-of-two head count n the geometric sequence 2^(-8/n), 2^(-16/n),
 * ... (8 heads: 1/2, 1/4, ..., 1/256).  For other counts: the sequence of the
 * largest power of two p below n, followed by every other member (the 1st,
 * 3rd, ...) of the sequence for 2p until n slopes exist.
 */
void orc_alibi_slopes(int n_heads, double *slopes)
{
    int p = 1;
    while (2 * p <= n_heads) p *= 2;
    for (int i = 0; i < p; ++i) slopes[i] = pow(2.0, -8.0 * (double)(i + 1) / (double)p);
    for (int i = 0; p + i < n_heads; ++i) slopes[p + i] = pow(2.0, -8.0 * (double)(2 * i + 1) / (double)(2 * p));
}

/*
 * Attention with the linear bias instead of a rotation:
 *   out[q][h][:] = sum_j softmax_j( Q[q][h] . K[j][kv(h)] / sqrt(d)  -  slope[h] (q_pos[q] - k_pos[j]) ) V[j][kv(h)]
 * over the keys j with k_pos[j] <= q_pos[q].  The paper asks for the bias to
 * follow the provided position IDs, so the distance is a difference of
 * position IDs, not of buffer rows: a module left out of the prompt leaves
 * its distance in place.  Q and K enter as they are (nothing is rotated).
 *
 * Q [nq][Hq][d]   K,V [nkv][Hkv][d]   slope [Hq]   out [nq][Hq][d]
 */
void orc_attn_alibi(const double *Q, const int32_t *q_pos, int nq, const double *K, const double *V,
                    const int32_t *k_pos, int nkv, int Hq, int Hkv, int d, const double *slope, double *out)
{
    int group = Hq / Hkv;
    double inv_sqrt_d = 1.0 / sqrt((double)d);
    long pairs = (long)nq * Hq;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 4) num_threads(g_threads)
#endif
    for (long w = 0; w < pairs; ++w) {
        int q = (int)(w / Hq), h = (int)(w % Hq);
        int kvh = h / group;
        const double *qv = Q + ((size_t)q * Hq + h) * d;
        double *s = (double *)malloc(sizeof(double) * (size_t)(nkv > 0 ? nkv : 1));
        for (int j = 0; j < nkv; ++j) {
            if (k_pos[j] <= q_pos[q]) {
                const double *k = K + ((size_t)j * Hkv + kvh) * d;
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += qv[c] * k[c];
                s[j] = dot * inv_sqrt_d - slope[h] * (double)(q_pos[q] - k_pos[j]);
            } else {
                s[j] = -INFINITY;
            }
        }
        softmax_times_v(s, nkv, V + (size_t)kvh * d, Hkv * d, d, out + ((size_t)q * Hq + h) * d);
        free(s);
    }
}

/* ------------------------------------------------------------------ */
/* Full recompute under module-local masking  (Sec. 3.1, Sec. 3.3)      */
/* ------------------------------------------------------------------ */

/*
 * The paper's equivalence: serving from cached modules equals running the
 * whole prompt in one pass with an attention mask that confines each module's
 * tokens to their own module.  This function is that one pass for a single
 * attention layer.
 *
 * All N tokens of the prompt (module tokens and uncached tokens, in any order)
 * come in raw; every Q and every K is rotated here at its own position ID.
 * Token a may attend token b iff
 *      pos[b] <= pos[a]   and   ( module_of[a] == module_of[b]  or  a is uncached ),
 * where uncached tokens carry module_of == -1.
 *
 * Q_raw [N][Hq][d]  K_raw,V [N][Hkv][d]  out [N][Hq][d]
 * K_enc (out, may be NULL) [N][Hkv][d]: the rotated keys, for comparing a
 * module's rows with that module encoded on its own.
 */
void orc_full_masked(const double *Q_raw, const double *K_raw, const double *V, const int32_t *pos,
                     const int32_t *module_of, int N, int Hq, int Hkv, int d, double base, double *out,
                     double *K_enc)
{
    int group = Hq / Hkv;
    double inv_sqrt_d = 1.0 / sqrt((double)d);
    double *Kr = (double *)malloc(sizeof(double) * (size_t)N * Hkv * d);
    double *Qr = (double *)malloc(sizeof(double) * (size_t)N * Hq * d);
    memcpy(Kr, K_raw, sizeof(double) * (size_t)N * Hkv * d);
    memcpy(Qr, Q_raw, sizeof(double) * (size_t)N * Hq * d);
    orc_rope(Kr, N, Hkv, d, pos, base);
    orc_rope(Qr, N, Hq, d, pos, base);
    if (K_enc) memcpy(K_enc, Kr, sizeof(double) * (size_t)N * Hkv * d);
    double *s = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    for (int a = 0; a < N; ++a) {
        for (int h = 0; h < Hq; ++h) {
            int kvh = h / group;
            const double *qa = Qr + ((size_t)a * Hq + h) * d;
            for (int b = 0; b < N; ++b) {
                int allowed = (pos[b] <= pos[a]) && (module_of[a] == module_of[b] || module_of[a] < 0);
                if (allowed) {
                    const double *kb = Kr + ((size_t)b * Hkv + kvh) * d;
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += qa[c] * kb[c];
                    s[b] = dot * inv_sqrt_d;
                } else {
                    s[b] = -INFINITY;
                }
            }
            softmax_times_v(s, N, V + (size_t)kvh * d, Hkv * d, d, out + ((size_t)a * Hq + h) * d);
        }
    }
    free(s);
    free(Qr);
    free(Kr);
}

/* ------------------------------------------------------------------ */
/* Parameterised modules  (Sec. 3.2.2; Sec. 3.3, last paragraph)        */
/* ------------------------------------------------------------------ */

/* Position ID of a buffer row that holds no token: larger than any query's,
 * so the rule  pos_k <= pos_q  never admits it. */
#define ORC_POS_NONE INT32_MAX

/*
 * A module was encoded with a parameter of `len` placeholder tokens; their
 * rows sit at K/V/pos[row0 .. row0+len) of an assembled buffer and already
 * carry the placeholders' position IDs.  A prompt supplies an argument of
 * n_arg <= len tokens.  Argument token i takes over the position ID of
 * placeholder i; its states replace the placeholder's: the key is the raw key
 * rotated at that position ID, the value is copied.  Placeholders beyond the
 * argument are white space that carries no meaning: they cease to be tokens
 * (their position becomes ORC_POS_NONE; their states are left as they are
 * and can never be seen).
 *
 * K,V   [rows][n_heads][d] assembled buffer (fp64), pos [rows]
 * K_arg_raw, V_arg  [n_arg][n_heads][d]
 * returns 0, or -1 when the argument is longer than the parameter.
 */
int orc_fill_param(double *K, double *V, int32_t *pos, int row0, int len, const double *K_arg_raw,
                   const double *V_arg, int n_arg, int n_heads, int d, double base)
{
    if (n_arg < 0 || len < 0 || n_arg > len) return -1;
    const size_t row = (size_t)n_heads * d;
    for (int i = 0; i < n_arg; ++i) {
        double *k = K + (size_t)(row0 + i) * row;
        double *v = V + (size_t)(row0 + i) * row;
        for (size_t c = 0; c < row; ++c) {
            k[c] = K_arg_raw[(size_t)i * row + c];
            v[c] = V_arg[(size_t)i * row + c];
        }
        orc_rope(k, 1, n_heads, d, &pos[row0 + i], base);
    }
    for (int i = n_arg; i < len; ++i) pos[row0 + i] = ORC_POS_NONE;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Memory per cached token  (Table 2)                                   */
/* ------------------------------------------------------------------ */

/* Bytes of K and V one token occupies across a model: 2 tensors x layers x
 * (kv heads x head_dim) x bytes per element.  With kv heads x head_dim equal
 * to the hidden size this is the closed form behind the paper's table. */
long orc_bytes_per_token(int n_layers, int n_kv_heads, int head_dim, int elem_bytes)
{
    return 2L * n_layers * n_kv_heads * head_dim * elem_bytes;
}
