/*
 * kvs.h - C ABI of the MI355X (gfx950) KVSlimmer KV-cache merge step.
 *
 * One call of kvs_step() takes one attention layer's cache from `len` to `budget` tokens per
 * unit, where a unit is one (sequence, KV head) pair:
 *
 *   score          attention of a window of recent queries over every cached Key
 *                  (Sec. 4.1, Eq. attn_def_vec: e_i = q k_i^T / sqrt(d_k), alpha = softmax(e),
 *                  o = sum_t alpha_t v_t), averaged over the G*W query rows of the unit into one
 *                  distribution alpha_bar and one output o_bar;
 *   select         the r = len - budget adjacent pairs (edges) with the smallest accumulated
 *                  attention mass alpha_bar[m] + alpha_bar[m+1] are merged in one parallel step
 *                  (Sec. 3.1, chunk-based compression; App. C, paragraph (i)); the first n_sink
 *                  tokens are always preserved (Sec. 5, implementation details);
 *   merge_compact  merged Key by the gradient-free closed form of Sec. 4.2 (Eq. kstar_final, with
 *                  the norms of the forward-only vectors c11, c22, c12 of Eqs. c11_def-c12_def,
 *                  including the off-diagonal coupling term), merged Value by summation
 *                  (Sec. 3.1, v* = v_m + v_{m+1}) together with the slot's cardinality.
 *
 * Conventions
 *   - Pointers marked HOST are read on the host during the call and may be freed afterwards.
 *     Pointers marked DEVICE are caller-owned device memory, 16-byte aligned, rows contiguous.
 *     The library never allocates or frees device memory, never synchronises the stream and keeps
 *     no state between calls.  All work is enqueued on `hip_stream` (a hipStream_t; NULL = default
 *     stream) and completes asynchronously.
 *   - The return value is the only error channel.  Every argument error is detected on the host
 *     before anything is launched; in that case nothing has been enqueued.
 *   - Outputs must not overlap inputs, each other or the workspace (KVS_ERR_ALIAS).
 *   - A unit with len <= budget is passed through unchanged: len output rows, counts = 1.
 *     Otherwise it produces exactly `budget` rows.  Rows of a unit beyond its output count are
 *     never written.
 *   - All accumulation is fp32; merged K/V are rounded once (nearest-even) to io_dtype.
 */
#ifndef KVS_H
#define KVS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVS_VERSION 300          /* major*10000 + minor*100 + patch */
#define KVS_MAX_Q_ROWS 1024      /* largest supported G*W */
#define KVS_MAX_DECODE_ROWS 64   /* largest G*W of kvs_decode_attention */
#define KVS_MAX_LEN (1 << 22)    /* largest supported cache length of one unit, in tokens */
#define KVS_STATIC_SCRATCH_BYTES (16u << 20)   /* workspace that kvs_step_static brings along, per GPU */

typedef enum {
  KVS_OK = 0,
  KVS_ERR_INVALID_ARG = 1,  /* null pointer, misaligned pointer, non-positive size, head_dim not 64/128,
                               G*W above KVS_MAX_Q_ROWS, overlapping units, unknown key_rule, causal not 0/1 */
  KVS_ERR_DTYPE = 2,        /* io_dtype is neither KVS_F32 nor KVS_BF16, or not the one the call supports */
  KVS_ERR_BUDGET = 3,       /* budget < n_sink + 1 + n_recent for a unit that has to merge (len > budget),
                               or budget < 1 */
  KVS_ERR_WORKSPACE = 4,    /* workspace null, misaligned (256 B) or smaller than kvs_workspace_size(); only the
                               calls that need one check it: for kvs_select and the kvs_merge_compact family it is
                               optional (see there; NULL and 0 are fine)                                 */
  KVS_ERR_ALIAS = 5,        /* an output overlaps an input, another output or the workspace */
  KVS_ERR_DEVICE = 6        /* a HIP launch failed.  The library reads the calling thread's HIP error state after
                               each launch (which clears it) and drops an error left pending by the caller's own
                               earlier HIP calls when a call starts; the cause is printed to stderr when the
                               testing switch KVS_DEBUG_VERBOSE (kvs_debug.h) is set                      */
} kvs_status;

typedef enum { KVS_F32 = 0, KVS_BF16 = 1 } kvs_dtype;

/* Rule for the merged Key of a slot of several rows (Values, cardinalities and slots do not depend on it). */
typedef enum {
  KVS_RULE_HESSIAN = 0,     /* Sec. 4.2, Eq. kstar_final: exact-Hessian weights with the off-diagonal coupling */
  KVS_RULE_DIAGONAL = 1,    /* ablation: the coupling blocks dropped (C_t := 0), weights proportional to A_t   */
  KVS_RULE_MEAN = 2         /* ablation: arithmetic mean over the tokens the rows stand for                    */
} kvs_key_rule;

typedef struct {
  int32_t n_units;          /* n_seq * n_kv_heads; one unit = one sequence's one KV head            */
  int32_t group;            /* G: query heads per KV head                                            */
  int32_t window;           /* W: recent queries per query head                                      */
  int32_t head_dim;         /* D = d_k = d_v; 64 or 128                                              */
  int32_t n_sink;           /* tokens [0, n_sink) are never merged (paper default 32)                */
  int32_t n_recent;         /* the last n_recent tokens are never merged (default 0)                 */
  kvs_dtype io_dtype;       /* dtype of Q, K, V, K_out, V_out                                        */
  float scale;              /* logit scale; 0 selects 1/sqrt(head_dim)                               */
  const int32_t* len;       /* HOST [n_units] cached tokens per unit (1 .. KVS_MAX_LEN)              */
  const int32_t* budget;    /* HOST [n_units] tokens to keep per unit                                */
  const int64_t* in_row;    /* HOST [n_units] first row of the unit in K, V, alpha_bar, edge_mask,
                               slot_of_token; the units' row ranges [in_row, in_row + len) must be
                               disjoint                                                              */
  const int64_t* out_row;   /* HOST [n_units] first row of the unit in K_out, V_out, counts_out;
                               ranges [out_row, out_row + min(len, budget)) must be disjoint         */
  kvs_key_rule key_rule;    /* KVS_RULE_HESSIAN (0) unless an ablation is wanted                     */
  int32_t causal;           /* 0: every query row attends to the whole cache.  1: causal mask inside the
                               window: the W queries of a head are those of the last W positions, whose
                               Keys and Values are the unit's last W rows, and the query at window position
                               w (row g*W + w of the unit's block of Q) attends to rows t <= len - W + w
                               only (Eq. attn_def_vec over that prefix).  Needs len >= window
                               (KVS_ERR_INVALID_ARG).  Read by kvs_score*, kvs_step*, kvs_sensitivity and
                               kvs_step_per_query; kvs_decode_attention ignores it.                     */
} kvs_problem;

/* Bytes of DEVICE workspace (256-byte aligned) that the calls below need for this problem. */
kvs_status kvs_workspace_size(const kvs_problem* p, size_t* bytes);

/* Sec. 4.1, Eq. attn_def_vec, averaged over the unit's query rows.
 *   Q         DEVICE [n_units, G, W, D] io_dtype
 *   K, V      DEVICE [rows, D] io_dtype; unit u occupies rows in_row[u] .. in_row[u]+len[u]-1
 *   alpha_bar DEVICE out [rows] fp32: mean over the G*W rows of softmax_t(scale * q.k_t)
 *   o_bar     DEVICE out [n_units, D] fp32: sum_t alpha_bar[t] V[t]                              */
kvs_status kvs_score(const kvs_problem* p, const void* Q, const void* K, const void* V,
                     float* alpha_bar, float* o_bar,
                     void* ws, size_t ws_bytes, void* hip_stream);

/* Sec. 3.1 (parallel merge of adjacent pairs back to the budget) with the ranking of App. C (i).
 *   edge score sigma[m] = alpha_bar[m] + alpha_bar[m+1], added and compared in fp32, for the eligible
 *   edges n_sink <= m <= len-2-n_recent; the r = len - budget smallest are selected, ties to the lower m.
 *   edge_mask     DEVICE out [rows] u8: 1 = token m+1 joins the slot of token m (last token: 0)
 *   slot_of_token DEVICE out [rows] i32: unit-local output slot of every token (non-decreasing)
 *   ws            optional.  With a workspace (256-byte aligned, at least kvs_workspace_size(p) bytes) a long unit's
 *                 selection may be spread over several workgroups that meet through it; with NULL, a misaligned or
 *                 a smaller one, every unit is selected by one workgroup, and a launch covers at most 64 units (with
 *                 one: up to 1024 short units).  The results are the same bit for bit. */
kvs_status kvs_select(const kvs_problem* p, const float* alpha_bar,
                      uint8_t* edge_mask, int32_t* slot_of_token,
                      void* ws, size_t ws_bytes, void* hip_stream);

/* Sec. 4.2, Eq. kstar_final (Keys) and Sec. 3.1, v* = v_m + v_{m+1} (Values), one pass over K and V.
 *   For a slot S of consecutive tokens: A_t = alpha_t |1 - 2 alpha_t| ||v_t - o||, C_t =
 *   alpha_t alpha_{t+1} ||v_t + v_{t+1} - 2o|| on the slot's inner edges, u_t = A_t - C_{t-1} - C_t,
 *   K_out[S] = sum u_t K[t] / sum u_t (arithmetic mean of the slot if that denominator is not a
 *   positive finite number), V_out[S] = sum V[t], counts_out[S] = |S|.  A slot of one token is a
 *   bit-exact copy.
 *   K_out, V_out DEVICE out [out rows, D] io_dtype;  counts_out DEVICE out [out rows] i32          */
/*   ws           optional (also for the _counts and _norms forms).  The kernel needs none; with a workspace (256-byte
 *                aligned, at least kvs_workspace_size(p) bytes) a call with more than 64 short units puts up to 1024 of
 *                them into one launch, whose unit descriptors then live there.  Same results either way.
 *   edge_mask and slot_of_token are taken as kvs_select writes them: slot_of_token[t] = number of zero mask bytes
 *   before t.  The mask byte of a unit's last token is read as 0 whatever it holds; a slot index outside the
 *   unit's output rows is never written.  Nothing else about a mask from outside the library is checked.   */
kvs_status kvs_merge_compact(const kvs_problem* p, const void* K, const void* V,
                             const float* alpha_bar, const float* o_bar,
                             const uint8_t* edge_mask, const int32_t* slot_of_token,
                             void* K_out, void* V_out, int32_t* counts_out,
                             void* ws, size_t ws_bytes, void* hip_stream);

/* score -> select -> merge_compact in one call; intermediates live in the workspace.
 *   slot_of_token_out, edge_mask_out: optional DEVICE outputs (NULL to keep them internal).       */
kvs_status kvs_step(const kvs_problem* p, const void* Q, const void* K, const void* V,
                    void* K_out, void* V_out, int32_t* counts_out,
                    int32_t* slot_of_token_out, uint8_t* edge_mask_out,
                    void* ws, size_t ws_bytes, void* hip_stream);

/* Streaming regime (Sec. 3.1, last paragraph; Sec. 5): the cache is compressed again whenever it has grown
 * past the budget by a chunk, so the input of a step is itself a merged cache.  Row t then is a slot
 * (k, V, c): c = counts_in[t] tokens that share the Key k and whose Values add up to V (what
 * kvs_merge_compact returns as K_out, V_out, counts_out).  Such a slot enters every formula as one token
 * with logit e + ln c and value V / c: alpha_bar[t] is the slot's total attention mass, o_bar = sum_t
 * alpha_bar[t] V[t] / c_t, the residual of the Key rule is V[t] / c_t - o_bar, merged Values stay sums,
 * counts_out[S] = sum of counts_in over the slot, and the fallback Key is the mean over the tokens the rows
 * stand for.  kvs_select is unchanged (it sees alpha_bar only).
 *   counts_in DEVICE in [rows] i32, every entry >= 1; NULL = plain tokens, i.e. exactly the calls above.
 * All other arguments, layouts, ownership and error behaviour are those of the calls above.              */
kvs_status kvs_score_counts(const kvs_problem* p, const void* Q, const void* K, const void* V,
                            const int32_t* counts_in, float* alpha_bar, float* o_bar,
                            void* ws, size_t ws_bytes, void* hip_stream);
kvs_status kvs_merge_compact_counts(const kvs_problem* p, const void* K, const void* V, const int32_t* counts_in,
                                    const float* alpha_bar, const float* o_bar,
                                    const uint8_t* edge_mask, const int32_t* slot_of_token,
                                    void* K_out, void* V_out, int32_t* counts_out,
                                    void* ws, size_t ws_bytes, void* hip_stream);
kvs_status kvs_step_counts(const kvs_problem* p, const void* Q, const void* K, const void* V, const int32_t* counts_in,
                           void* K_out, void* V_out, int32_t* counts_out,
                           int32_t* slot_of_token_out, uint8_t* edge_mask_out,
                           void* ws, size_t ws_bytes, void* hip_stream);

/* For callers that cannot allocate device memory or keep a workspace around: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  kvs_step_counts (counts_in = NULL: kvs_step) without the
 * workspace arguments: the intermediates live in a device array of KVS_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (every GPU the library runs on holds one copy until the process ends).  The call
 * allocates and frees nothing, on the device or through any allocating runtime routine, and never synchronises.
 *   - A problem whose kvs_workspace_size() exceeds KVS_STATIC_SCRATCH_BYTES is refused with KVS_ERR_WORKSPACE
 *     before anything is launched (one layer of 8 KV heads x 32768 tokens, 128 query rows, needs about 3.1 MB).
 *   - The device of hip_stream must be the calling thread's current device.  The first call on a device looks
 *     up that device's copy of the array (hipGetSymbolAddress): make it outside a graph capture.
 *   - All calls on one GPU share the one array: two calls that may overlap in time (different streams, or one
 *     stream per thread) race.  Calls on one stream are ordered and may follow each other freely; nothing in
 *     the array has to survive from one call to the next or to start at zero.
 * Arguments, outputs, layouts and every other error are those of kvs_step_counts.                          */
kvs_status kvs_step_static(const kvs_problem* p, const void* Q, const void* K, const void* V, const int32_t* counts_in,
                           void* K_out, void* V_out, int32_t* counts_out,
                           int32_t* slot_of_token_out, uint8_t* edge_mask_out, void* hip_stream);

/* Sec. 3.1 (sum-merged Values with cardinality normalisation): attention of the problem's G*W query rows
 * over a merged cache, the consumer of kvs_merge_compact's outputs.  Row t of unit u (rows in_row[u] ..
 * in_row[u] + len[u] of K, V, counts) is a slot (k', V', c) standing for c tokens with the Key k' whose
 * Values add up to V':
 *   out[u, q, :] = sum_t exp(e_t) V[t] / sum_t counts[t] exp(e_t),   e_t = scale * Q[u, q] . K[t]
 * which is attention over the tokens the rows stand for.  budget, n_sink, n_recent and key_rule of the
 * problem are not used (pass budget = len); G*W <= KVS_MAX_DECODE_ROWS (KVS_ERR_INVALID_ARG above).
 *   Q       DEVICE in  [n_units, G, W, D] io_dtype
 *   K, V    DEVICE in  [rows, D] io_dtype (for example K_out, V_out of a merge step)
 *   counts  DEVICE in  [rows] i32, or NULL for a cache of plain tokens
 *   out     DEVICE out [n_units, G*W, D] fp32
 *   ws      DEVICE workspace of kvs_decode_workspace_size(p) bytes, 256-byte aligned (KVS_ERR_WORKSPACE)
 * Asynchronous on hip_stream; nothing is allocated; errors are found on the host before any launch.     */
kvs_status kvs_decode_workspace_size(const kvs_problem* p, size_t* bytes);
kvs_status kvs_decode_attention(const kvs_problem* p, const void* Q, const void* K, const void* V,
                                const int32_t* counts, float* out,
                                void* ws, size_t ws_bytes, void* hip_stream);

/* Per-query aggregation: an alternative to averaging the query rows' attention before the Key rule.
 * Sec. 4 derives c_tt = alpha_t (1 - 2 alpha_t)(v_t - o) and c_{t,t+1} = -alpha_t alpha_{t+1}(v_t + v_{t+1} - 2o)
 * (Eqs. c11_def-c12_def) for one query.  Here every query row q of the unit keeps its own attention
 * alpha^{(q)} = softmax_t(scale * Q[q].K[t]) and its own output o^{(q)} = sum_t alpha^{(q)}_t V[t] (Eq.
 * attn_def_vec), and the norms are averaged over the G*W rows:
 *   A_t = mean_q alpha^{(q)}_t |1 - 2 alpha^{(q)}_t| ||v_t - o^{(q)}||
 *   C_t = mean_q alpha^{(q)}_t alpha^{(q)}_{t+1} ||v_t + v_{t+1} - 2 o^{(q)}||      (edge t, t+1)
 * kvs_merge_compact_norms is kvs_merge_compact with these A and C in u_t = A_t - C_{t-1} - C_t (Eq.
 * kstar_final); Values, cardinalities, key_rule and the fallback are as there.  The partition still comes from
 * kvs_select on alpha_bar.  With one query row the results are those of the calls above.
 * Restrictions: with io_dtype KVS_BF16 every unit has at least 32 rows (KVS_ERR_INVALID_ARG; the matrix-core
 * kernels work on whole tiles), with KVS_F32 any length is taken (vector-ALU kernels, written for the small
 * configurations, not for speed).  kvs_merge_compact_norms takes both dtypes and any length.
 * The *_counts forms take the input rows' cardinalities (streaming regime, as kvs_step_counts; NULL = the plain
 * call): every query row then sees row t as one token with logit e + ln counts_in[t] and value
 * V[t] / counts_in[t], and the merge adds the cardinalities up.
 *   alpha_bar DEVICE out [rows] fp32, as from kvs_score
 *   a_tok     DEVICE out / in [rows] fp32: A_t
 *   c_edge    DEVICE out / in [rows] fp32: C_t; the entry of a unit's last row is 0 and never read
 *   ws        DEVICE workspace of kvs_per_query_workspace_size(p) bytes, 256-byte aligned (kvs_sensitivity,
 *             kvs_step_per_query; kvs_merge_compact_norms uses none)
 * All other arguments, layouts, ownership and error behaviour are those of kvs_score, kvs_merge_compact and
 * kvs_step.                                                                                                   */
kvs_status kvs_per_query_workspace_size(const kvs_problem* p, size_t* bytes);
kvs_status kvs_sensitivity(const kvs_problem* p, const void* Q, const void* K, const void* V,
                           float* alpha_bar, float* a_tok, float* c_edge,
                           void* ws, size_t ws_bytes, void* hip_stream);
kvs_status kvs_merge_compact_norms(const kvs_problem* p, const void* K, const void* V,
                                   const float* a_tok, const float* c_edge,
                                   const uint8_t* edge_mask, const int32_t* slot_of_token,
                                   void* K_out, void* V_out, int32_t* counts_out,
                                   void* ws, size_t ws_bytes, void* hip_stream);
kvs_status kvs_step_per_query(const kvs_problem* p, const void* Q, const void* K, const void* V,
                              void* K_out, void* V_out, int32_t* counts_out,
                              int32_t* slot_of_token_out, uint8_t* edge_mask_out,
                              void* ws, size_t ws_bytes, void* hip_stream);
kvs_status kvs_sensitivity_counts(const kvs_problem* p, const void* Q, const void* K, const void* V,
                                  const int32_t* counts_in, float* alpha_bar, float* a_tok, float* c_edge,
                                  void* ws, size_t ws_bytes, void* hip_stream);
kvs_status kvs_merge_compact_norms_counts(const kvs_problem* p, const void* K, const void* V,
                                          const int32_t* counts_in, const float* a_tok, const float* c_edge,
                                          const uint8_t* edge_mask, const int32_t* slot_of_token,
                                          void* K_out, void* V_out, int32_t* counts_out,
                                          void* ws, size_t ws_bytes, void* hip_stream);
kvs_status kvs_step_per_query_counts(const kvs_problem* p, const void* Q, const void* K, const void* V,
                                     const int32_t* counts_in, void* K_out, void* V_out, int32_t* counts_out,
                                     int32_t* slot_of_token_out, uint8_t* edge_mask_out,
                                     void* ws, size_t ws_bytes, void* hip_stream);

const char* kvs_status_str(kvs_status s);
int kvs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVS_H */
