/*
 * ltri.h — C ABI of libltri: the per-chunk streaming sparse-attention step of
 * Ltri-LLM on one AMD MI355X (gfx950).
 *
 * The three verbs follow the paper's three steps (Sec. 3.4 "Overall Framework"):
 *   step 1  ltri_append_chunk   segment the new tokens into spans at the borders of the
 *                               triangular regions of their attention map (Sec. 3.2,
 *                               Eq. 1-5, NMS; appendix "NMS Input Filtration") and store
 *                               one representative key per span (Sec. 3.3.1);
 *   step 2  ltri_retrieve       score the stored spans against the query chunk's span
 *                               representatives (Eq. 8) and pick the top spans (Eq. 9);
 *   step 3  ltri_attend         exact attention of the query chunk over
 *                               initial | retrieved | window | current tokens.
 *   all     ltri_step           the three in one call: fused kernels on one stream when the
 *                               keys and values are resident on the device; with evicted rows
 *                               in host memory the part of step 3 that does not depend on
 *                               step 2 runs beside the fetch of the retrieved rows, which a
 *                               second stream carries.
 *
 * Conventions
 *   - Every function returns an int32 status: 0 = LTRI_OK, negative = error. Nothing
 *     throws. ltri_strerror() names a status, ltri_last_error() gives the detail text
 *     of the last failing call on a context.
 *   - "device" pointers are HIP device addresses of the current device, "host" pointers
 *     are ordinary process memory. The library never allocates or frees device memory:
 *     the caller sizes buffers with ltri_workspace_bytes(), allocates them (with any
 *     allocator) and keeps them alive until ltri_destroy(). The library owns only the
 *     host-side ltri_ctx.
 *   - All device work is enqueued on the stream given at creation and the call returns
 *     without waiting, except the introspection calls marked "synchronises". With kv_offload
 *     ltri_step also uses a second stream and two events that the context creates and owns; its
 *     results are ordered on the context's stream like everyone else's.
 *   - Tensors are dense, row-major, in the configured dtype (fp32 or bf16):
 *       KV arenas  [n_layers][n_seqs][n_kv_heads][max_tokens][head_dim]
 *       queries    [seq_count][n_q][n_q_heads][head_dim]
 *       outputs    [seq_count][n_q][n_q_heads][head_dim]
 *     Query head g belongs to KV head g / (n_q_heads / n_kv_heads).
 *   - Calls on one context must not overlap (one scratch buffer, one index memory), with one
 *     exception: ltri_append_chunk for chunk t+1 touches nothing that ltri_attend for chunk t
 *     reads, so the two may run concurrently on different streams (see ltri_set_stream); the
 *     caller orders append(t+1) after retrieve(t) and retrieve(t+1) after append(t+1).
 */
#ifndef LTRI_H
#define LTRI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define LTRI_OK          0
#define LTRI_EINVAL     -1   /* bad argument / unsupported configuration            */
#define LTRI_ESTATE     -2   /* calls out of order (e.g. retrieve before append)     */
#define LTRI_ECAPACITY  -3   /* token or span capacity exceeded                       */
#define LTRI_EHIP       -4   /* a HIP runtime call failed                             */

/* dtypes */
#define LTRI_F32   0
#define LTRI_BF16  1

/* kinds of segmentation map */
#define LTRI_MAP_SOFTMAX 0   /* Eq. 1-3: causal softmax over the chunk's own keys      */
#define LTRI_MAP_LOGIT   1   /* masked scaled scores q.k/sqrt(d), no softmax           */

/* representative vector of a span */
#define LTRI_REP_MEAN    0   /* mean of the span's rows (Sec. 3.3.1, mean pooling)     */
#define LTRI_REP_DYNAMIC 1   /* dynamic span index vectors (Sec. 3.3.2), see ltri_config */
#define LTRI_RATIO_ROW    0  /* area ratio of a span against its row neighbours (the paper's default) */
#define LTRI_RATIO_COL    1  /* ... against its column neighbours                        */
#define LTRI_RATIO_ROWCOL 2  /* ... against both                                         */

#define LTRI_MAX_BATCH   64  /* most sequences one call can take                        */

typedef struct ltri_ctx ltri_ctx;

typedef struct {
  int32_t n_q_heads, n_kv_heads, head_dim;  /* head_dim 64 or 128 (bf16: 128 only)       */
  int32_t dtype;                            /* LTRI_F32 | LTRI_BF16                       */
  int32_t n_layers, n_seqs;
  int64_t max_tokens;                       /* capacity per sequence                      */
  int32_t chunk_max;                        /* most tokens one append may bring, <= 2048  */
  int32_t n_sink, window;                   /* initial tokens, local window               */
  int32_t k_max;                            /* cap on retrieved spans, 0 = none           */
  int64_t budget_tokens;                    /* cap on retrieved tokens, 0 = none          */
  int32_t seg_map;                          /* LTRI_MAP_*                                 */
  float   theta, phi;                       /* Eq. 5 threshold (absolute, per head and
                                               cell); NMS IoU threshold                   */
  int32_t max_spans_per_chunk;              /* cap on NMS keeps per chunk, 0 = none       */
  int32_t rep_mode;                         /* LTRI_REP_MEAN | LTRI_REP_DYNAMIC           */
  int32_t max_spans;                        /* span capacity per (layer, seq, KV head);
                                               0 = max_tokens / 32 + 64                   */
  /* LTRI_REP_DYNAMIC only (Sec. 3.3.2). Votes v_x (Eq. 6) are the column sums of the chunk's
   * head-summed softmax map; r_a is the area of a span's triangle over that area plus its
   * neighbours' (ratio_mode); the span keeps round(len / e^(lambda (1 - r_a))) index tokens
   * (Eq. 7; ties to even), at least index_min, at most index_max (0 = no limit), between 1 and
   * len: the tokens with the most votes, earlier ones first on ties. One vector per span is
   * stored, the sum of the keys of its index tokens (Eq. 8 is bilinear); the query side of
   * step 2 sums the group's query rows over the same tokens of the chunk. */
  float   lambda;
  int32_t index_min, index_max;
  int32_t ratio_mode;                       /* LTRI_RATIO_*                               */
  /* > 0: the threshold of Eq. 5 is this percentile of the chunk's map (Sec. 4, "Hyperparameter
   * Tuning": typically the 90th, i.e. 0.9): the value of rank floor(q (n - 1)) among the n
   * cells on and below the diagonal of the head-summed map, per head-summed cell; `theta` is
   * then ignored. Must be below or equal to 1. */
  float   theta_quantile;
  /* > 0: retrieval by memory units as in Eq. 9. The stream is cut into units (blocks) of this
   * many tokens at absolute positions; spans are also cut at unit edges, a unit scores the
   * maximum over its spans, and step 2 orders units by (-score, id) and takes the longest prefix
   * within k_max units and budget_tokens evicted tokens; selections (sel_ids, forced and
   * persistent ones) then hold unit ids and the context set holds whole units' evicted parts.
   * At most chunk_max, and max_tokens / unit_tokens + 1 <= 8192. 0: spans are retrieved. */
  int32_t unit_tokens;
  /* 1: host-offloaded KV (Sec. 3.4 first step: the keys and values of evicted tokens live in CPU memory, only
   * their index vectors stay on the GPU). k_arena / v_arena given to ltri_create are then HOST arenas of the
   * usual layout in pinned, device-visible memory (hipHostMalloc, or torch's pin_memory): every appended row is
   * written there. On the device the context keeps, inside `state`, per (layer, sequence, KV head) only the
   * initial tokens, a ring of the latest tokens (a power of two >= window + 2 chunk_max rows) and room for the
   * rows of one selection; step 2 ends by fetching the selected tokens' rows from the host arenas into that room
   * (a kernel reading host memory; no host synchronisation), and step 3 reads initial | fetched | ring rows.
   * Results are those of the resident layout bit for bit. The chunk's rows must be passed to the append
   * (k_chunk / v_chunk non-NULL). 0: everything resident in the device arenas. */
  int32_t kv_offload;
  /* > 0, with LTRI_REP_DYNAMIC and unit_tokens > 0: the paper's M (Sec. 4, "Compression Ratio": up to M span
   * index vectors per block of 128 tokens; 12 or 24 in its configurations). A block is the part of a memory unit
   * that lies in the appended chunk. If the Eq. 7 counts of a block's spans (after index_min / index_max) add up
   * to more than M, the largest are levelled down: every span keeps min(count, level) for the highest level that
   * fits, and what is left of M goes, one vector each, to the earliest spans still below their own count; no
   * span drops below one. 0: no block budget. EINVAL without dynamic index vectors or without units. */
  int32_t index_block_max;
} ltri_config;

/* Sizes (bytes) of the two device buffers a context needs: `state` holds the index
 * memory (span table, representative keys, selections, token lists; lives as long as
 * the context; ltri_create enqueues a kernel that zero-fills it), `scratch` holds per-call
 * temporaries. EINVAL on an unsupported configuration. */
int32_t ltri_workspace_bytes(const ltri_config* cfg, size_t* state_bytes, size_t* scratch_bytes);

/* Creates a context. k_arena / v_arena / state / scratch are device pointers owned by the
 * caller (256-byte aligned; with kv_offload the two arenas are pinned host memory instead),
 * hip_stream is a hipStream_t (NULL = default stream). The call enqueues a kernel that clears `state`. */
int32_t ltri_create(const ltri_config* cfg, void* k_arena, void* v_arena, void* state, void* scratch,
                    void* hip_stream, ltri_ctx** out);
int32_t ltri_destroy(ltri_ctx* ctx);
/* Forget all layers of one sequence (span table, selections, token count). */
int32_t ltri_reset(ltri_ctx* ctx, int32_t seq);
/* Stream on which the following calls enqueue their work (hipStream_t; NULL = default stream).
 * Ordering between work on different streams is the caller's business (events). */
int32_t ltri_set_stream(ltri_ctx* ctx, void* hip_stream);
/* LDS ring depth of the bf16 attention kernel: 4 (default, 130 KB of LDS per compute unit, fastest
 * on its own) or 3 (98 KB, leaves room for the segmentation kernels of the next chunk to run next
 * to it). EINVAL otherwise. */
int32_t ltri_set_attend_stages(ltri_ctx* ctx, int32_t stages);
/* A context without device buffers: every call validates its arguments and advances the
 * host-side state exactly as a real context would, but enqueues nothing; introspection calls
 * return ESTATE. Used to test the host logic on a machine without a GPU. */
int32_t ltri_create_dry(const ltri_config* cfg, ltri_ctx** out);

/* Step 1 (Sec. 3.4 first step; Sec. 3.2; Sec. 3.3.1). For each sequence s in
 * [seq_begin, seq_begin + seq_count): tokens [T_s, T_s + n_new) of `layer` are appended.
 *   k_chunk, v_chunk  device [seq_count][n_kv_heads][n_new][head_dim], copied into the
 *                     arenas first; both NULL = the caller already wrote them in place.
 *   q_seg             device [seq_count][n_new][n_q_heads][head_dim]: queries whose map is
 *                     segmented (Eq. 1), summed over each KV head's group (Eq. 4); NULL =
 *                     the keys are used as queries (one head per KV head).
 * The chunk's causal map is scored (Eq. 4-5), the best span on every anti-diagonal is kept
 * if its score is > 0 (ties: shorter span), greedy NMS on 1-D token intervals with IoU
 * threshold phi removes overlaps (ties: smaller start, then smaller end), the kept
 * intervals' end points cut the chunk into consecutive spans, and every span's mean key is
 * stored, rounded once to the dtype.
 * ECAPACITY if T_s + n_new > max_tokens; EINVAL if n_new < 1 or > chunk_max. Overflow of
 * the span table is detected on the device and reported by ltri_sync_status(). */
int32_t ltri_append_chunk(ltri_ctx* ctx, int32_t layer, int32_t seq_begin, int32_t seq_count,
                          const void* k_chunk, const void* v_chunk, const void* q_seg, int32_t n_new);

/* Same for one sequence, with the span boundaries supplied by the caller instead of
 * segmenting: bounds_host holds, for each KV head h, n_bounds_host[h] strictly increasing
 * chunk-local offsets, the first 0 and the last n_new, heads back to back. */
int32_t ltri_append_chunk_with_spans(ltri_ctx* ctx, int32_t layer, int32_t seq,
                                     const void* k_chunk, const void* v_chunk, int32_t n_new,
                                     const int32_t* bounds_host, const int32_t* n_bounds_host);

/* Step 2 (Sec. 3.4 second step, Eq. 8-9). q: device [seq_count][n_q][n_q_heads][head_dim],
 * the queries of the chunk appended last (n_q must equal its length, else ESTATE).
 * Per KV head: query-span representatives = mean over each of the chunk's spans of the
 * group-summed queries; score of a stored span = max over query spans of the dot product
 * with its representative key; spans that reach into the evicted region
 * [n_sink, chunk_start - window) are eligible and count with their part inside it; they
 * are ordered by (-score, id) and the longest prefix with at most k_max spans and at most
 * budget_tokens tokens is selected. The ascending ids are kept in the context and, if
 * sel_ids / sel_cnt are not NULL, also written to device [seq_count][n_kv_heads][sel_cap]
 * and [seq_count][n_kv_heads] (sel_cap from ltri_sel_capacity()). */
int32_t ltri_retrieve(ltri_ctx* ctx, int32_t layer, int32_t seq_begin, int32_t seq_count,
                      const void* q, int32_t n_q, int32_t* sel_ids, int32_t* sel_cnt);
int32_t ltri_sel_capacity(const ltri_ctx* ctx);

/* LTRI_REP_DYNAMIC, introspection (synchronises the stream): the index tokens of the chunk
 * appended last to (layer, seq, kv_head) as a bit mask, bit t of word t / 32 = token t of the
 * chunk; mask_host holds cap_words words, at least (chunk length + 31) / 32. ESTATE in a dry
 * context or when the context stores mean representatives. */
int32_t ltri_get_index_tokens(ltri_ctx* ctx, int32_t layer, int32_t seq, int32_t kv_head,
                              uint32_t* mask_host, int32_t cap_words);

/* theta_quantile > 0, introspection (synchronises the stream): the threshold that the segmentation of the chunk
 * appended last used for (layer, seq, kv_head), i.e. the cell of rank floor(q (n - 1)) of the chunk's head-summed
 * map in ascending order (Sec. 4, "Hyperparameter Tuning": the threshold as a percentile of the map). The device
 * keeps it only for the sequences of the last segmentation launch (up to four sequences of the last
 * ltri_append_chunk / ltri_step call, the last ones of a larger batch). ESTATE in a dry context, without
 * theta_quantile, for a one-token chunk, or for another layer or sequence than those. */
int32_t ltri_get_theta(ltri_ctx* ctx, int32_t layer, int32_t seq, int32_t kv_head, double* theta_host);

/* Collaborative voting (Sec. 3.5, Collaborative Voting), with retrieval by memory units
 * (unit_tokens > 0, EINVAL otherwise). Step 2 of `layer` in which the earlier layers take part:
 * the layer first selects units on its own as ltri_retrieve does; then every earlier layer l with
 * layer_weights_host[l] > 0 gives that weight to each unit of its current selection (same
 * sequence, same KV head index) and the layer gives layer_weights_host[layer] to each unit of its
 * own; eligible units are ordered by (votes descending, own score descending, id ascending) and
 * the longest prefix within k_max units and budget_tokens evicted tokens becomes the layer's
 * selection. Votes are float32 sums, earlier layers in ascending order, the layer last.
 * layer_weights_host: host array of at least layer + 1 non-negative weights (the paper uses the
 * retrieval-head scores of the layers that have a retrieval head, 0 elsewhere). ESTATE if a
 * voting layer has no selection for the same chunk of the sequence; EINVAL if max_tokens /
 * unit_tokens + 1 exceeds 4096. Other arguments as ltri_retrieve. */
int32_t ltri_retrieve_collaborative(ltri_ctx* ctx, int32_t layer, int32_t seq_begin, int32_t seq_count,
                                    const void* q, int32_t n_q, const float* layer_weights_host,
                                    int32_t* sel_ids, int32_t* sel_cnt);

/* Persistent selection (Sec. 3.5, Persistent Mechanism): step 2 without scoring. The span ids
 * selected by the most recent ltri_retrieve / ltri_force_selection of each (sequence, KV head)
 * are kept, and the context set of the last appended chunk is rebuilt from them: initial
 * tokens, the kept spans' parts inside the evicted region as it is now, the window. Meant for
 * decoding with the evidence found by the last prefill chunk. No device arguments; work is
 * enqueued on the context's stream. ESTATE if a sequence has no chunk or never had a
 * selection since its last reset. */
int32_t ltri_retrieve_persistent(ltri_ctx* ctx, int32_t layer, int32_t seq_begin, int32_t seq_count);

/* Replace the selection of one KV head by ids_host[0..n) (stored span ids, any order,
 * ineligible ones contribute no tokens). Test seam and "mandatory injection". */
int32_t ltri_force_selection(ltri_ctx* ctx, int32_t layer, int32_t seq, int32_t kv_head,
                             const int32_t* ids_host, int32_t n);

/* Step 3 (Sec. 3.4 third step). out: device [seq_count][n_q][n_q_heads][head_dim] in the
 * dtype; lse: device fp32 [seq_count][n_q][n_q_heads] (natural-log sum of exponentials of
 * the scaled scores) or NULL. Query row i of the chunk attends the initial tokens, the
 * selected spans' evicted parts, the window and the chunk's tokens 0..i, with weights
 * softmax(q.k / sqrt(head_dim)). ESTATE unless ltri_retrieve (or ltri_force_selection for
 * every head) ran for this chunk. */
int32_t ltri_attend(ltri_ctx* ctx, int32_t layer, int32_t seq_begin, int32_t seq_count,
                    const void* q, int32_t n_q, void* out, float* lse);

/* ltri_attend for callers that cannot allocate device memory and bring no scratch for this call: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments, same
 * results. Where ltri_attend keeps the partial results of a split key range (query blocks of 1 to 4 rows:
 * decoding) in the context's scratch buffer, this call keeps them in a buffer of 2 MiB that the library
 * itself holds on every GPU it runs on, from load until the process ends. The call allocates and frees
 * nothing. LTRI_ECAPACITY if the partial results of this call need more than 2 MiB (they take
 * seq_count * n_q_heads * splits * n_q * (head_dim + 2) * 4 bytes; 16 sequences of one token at 32 query
 * heads take 1.1 MB); other errors as ltri_attend. All contexts on one GPU share the buffer: calls that
 * overlap on one GPU (different streams or contexts) race; on one stream they are ordered. Nothing in the
 * buffer has to start at zero, every word a call reads was written by that call. */
int32_t ltri_attend_static(ltri_ctx* ctx, int32_t layer, int32_t seq_begin, int32_t seq_count,
                           const void* q, int32_t n_q, void* out, float* lse);

/* One whole step of the path for one chunk (Sec. 3.4, the three steps): the same results as
 * ltri_append_chunk(k_chunk, v_chunk, q_seg) + ltri_retrieve(q) + ltri_attend(q), arguments as there
 * (k_chunk / v_chunk may both be NULL when the rows are already in the arenas; q_seg and lse may be
 * NULL; the selection is not copied out, read it with ltri_get_selection).
 * What this call adds is the schedule, which depends on where the evicted keys and values live.
 * Resident on the device (kv_offload = 0): the kernels of the three steps follow each other on the context's
 * stream without a return to the host. With mean representatives in bf16 (head_dim 128) step 2 is one launch:
 * running sums of the chunk's query and key rows, which need no span boundaries, are taken by further workgroups
 * of step 1's last launch, and step 2 forms Q^R of every query span and the mean keys of the chunk's spans as
 * differences of two of their rows before it scores, selects and writes the lists. Other configurations sum the
 * rows per span in a launch of their own. The attention is one launch over initial | retrieved | window |
 * chunk; results identical to the three calls.
 * In host memory (kv_offload = 1): the fetch of the retrieved rows over the host link is the longest part of the
 * step. It is queued on a second stream the context owns, behind step 2; the attention over initial tokens,
 * window and the chunk itself, which needs none of those rows, follows step 2 on the context's stream and runs
 * beside the fetch. The attention over the retrieved tokens follows on the context's stream once the fetch is
 * done, and folds the first part's output in by the two log-sum-exps as it writes. The context's stream waits
 * for the second stream before that launch, so for the caller everything is ordered on the context's stream as
 * with the three calls: `out` and `lse` hold the result once that stream reaches the end of this call's work.
 * The first part is rounded to the dtype before it is folded in, so `out` can differ from ltri_attend's by one
 * more rounding of the dtype.
 * A one-token chunk (decode) runs steps 1 and 2 in one kernel launch and then step 3, all on the context's
 * stream, with results identical to the three calls. Chunks of 2 to 4 rows, fp32 contexts and group sizes the
 * matrix-core kernel does not take run the three calls in order.
 * Errors: those of the three calls. */
int32_t ltri_step(ltri_ctx* ctx, int32_t layer, int32_t seq_begin, int32_t seq_count, const void* k_chunk,
                  const void* v_chunk, const void* q_seg, const void* q, int32_t n_new, void* out, float* lse);

/* Measurement aid for ltri_step (Sec. 3.4 third step, the attention, is where the time goes): with timing on,
 * every ltri_step of a chunk of more than 4 rows on a bf16 context records HIP events around its attention
 * launches, on the context's stream. ltri_read_step_timing synchronises that stream,
 * writes two durations (milliseconds) per step for up to `cap` steps since the last read, oldest first, to the
 * host arrays, sets *n to the count and forgets the records. With resident keys and values the first array
 * holds the one attention launch (two events per step, carried by the launch's own dispatch: they take the
 * kernel's start and end) and the second 0; with kv_offload = 1 the first holds the launch over initial | window
 * | chunk (which shares the chip with the fetch) and the second the launch over the retrieved rows. Steps that run the plain calls (one-token chunks, fp32) leave no record. Turning timing on or off also
 * forgets pending records. */
int32_t ltri_set_step_timing(ltri_ctx* ctx, int32_t on);
int32_t ltri_read_step_timing(ltri_ctx* ctx, float* local_ms_host, float* retrieved_ms_host, int32_t cap, int32_t* n);

/* The gather on its own (Sec. 3.4 third step: the keys and values of the initial tokens, the retrieved
 * tokens and the local window are concatenated before the attention): copies the K and V rows of the
 * attended context set (initial | retrieved | window, in that order) of every KV head of one sequence into
 * k_packed / v_packed, device [n_kv_heads][list_cap][head_dim] (list_cap from
 * ltri_list_capacity()); n_tokens: device int32 [n_kv_heads] or NULL. */
int32_t ltri_gather_pack(ltri_ctx* ctx, int32_t layer, int32_t seq, void* k_packed, void* v_packed,
                         int32_t* n_tokens);
int32_t ltri_list_capacity(const ltri_ctx* ctx);

/* Introspection; these synchronise the stream. */
int32_t ltri_sync_status(ltri_ctx* ctx);   /* LTRI_OK or the first error raised on the device */
int32_t ltri_token_count(ltri_ctx* ctx, int32_t layer, int32_t seq, int64_t* n);
int32_t ltri_span_count(ltri_ctx* ctx, int32_t layer, int32_t seq, int32_t kv_head, int32_t* n);
int32_t ltri_get_spans(ltri_ctx* ctx, int32_t layer, int32_t seq, int32_t kv_head,
                       int32_t* starts_host, int32_t* lens_host, int32_t cap);
/* reps_host: [cap][head_dim] in the dtype. */
int32_t ltri_get_rep_keys(ltri_ctx* ctx, int32_t layer, int32_t seq, int32_t kv_head,
                          void* reps_host, int32_t cap);
/* Selection of the last retrieve: ids_host[cap], *n = count; scores_host (may be NULL):
 * fp64 score of every stored span, [span count]. */
int32_t ltri_get_selection(ltri_ctx* ctx, int32_t layer, int32_t seq, int32_t kv_head,
                           int32_t* ids_host, int32_t cap, int32_t* n, double* scores_host);
/* Context token list of the last retrieve: tokens_host[cap], *n = length. */
int32_t ltri_get_token_list(ltri_ctx* ctx, int32_t layer, int32_t seq, int32_t kv_head,
                            int32_t* tokens_host, int32_t cap, int32_t* n);

const char* ltri_strerror(int32_t status);
const char* ltri_last_error(const ltri_ctx* ctx);
/* "libltri <version> gfx950" */
const char* ltri_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LTRI_H */
