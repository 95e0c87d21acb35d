// Internal declarations shared by the host API and the HIP kernels of libltri.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "ltri.h"

namespace ltri {

// ---- per-slot metadata words (slot = (layer * n_seqs + seq) * n_kv_heads + kv_head) ----
enum : int {
  META_N_SPANS = 0,      // spans stored so far
  META_CHUNK_FIRST = 1,  // id of the first span of the chunk appended last
  META_CHUNK_NSP = 2,    // number of spans of that chunk
  META_CHUNK_START = 3,  // absolute position of that chunk's first token
  META_CHUNK_LEN = 4,    // its length
  META_SEL_CNT = 5,      // spans selected by the last retrieve
  META_LIST_LEN = 6,     // tokens in the context list (initial | retrieved | window)
  META_RESERVED = 7,
  META_WORDS = 8
};

constexpr int SEG_TB = 64;          // side of a segmentation tile
constexpr int SEG_MAX_L = 2048;     // longest chunk the segmentation kernels take
constexpr int SEG_MAX_NB = SEG_MAX_L / SEG_TB;
constexpr int SEG_MAX_DIAG = 2 * SEG_MAX_L;   // anti-diagonals of the largest map (2 L - 1), rounded up
constexpr int QUANT_BITS = 11;               // digit width of the radix selection of the percentile theta
constexpr int QUANT_BINS = 1 << QUANT_BITS;
constexpr int QUANT_LISTS = 16;               // sub-lists per problem (a tile appends to list tile % 16: fewer atomics per counter)
constexpr int QUANT_STATE_WORDS = 8 + QUANT_LISTS;   // per problem: key prefix, rank to go, theta (double bits), status, -, -, -, -, list lengths
constexpr int QUANT_LIST_CAP = 1 << 14;      // cells collected for the final exact selection, at most
constexpr int IDX_MASK_WORDS = SEG_MAX_L / 32;   // one bit per token of a chunk
constexpr int ATT_BN = 64;               // keys per attention tile; token lists are padded to it
constexpr int ATT_MAX_SPLITS = 16;       // key-range splits of a short query block (decode)
constexpr int ATT_SPLIT_MAX_ROWS = 4;    // longest query block that is split
constexpr size_t ATT_STATIC_SCRATCH_BYTES = 2u << 20;   // the library's own buffer for such partial results (ltri_attend_static)

// Byte offsets of the arrays inside the caller's `state` buffer.
struct StateLayout {
  size_t meta;        // int32  [n_slots][META_WORDS]
  size_t span_start;  // int32  [n_slots][max_spans]
  size_t span_len;    // int32  [n_slots][max_spans]
  size_t krep;        // dtype  [n_slots][max_spans][d]
  size_t scores;      // double [n_slots][max_spans]
  size_t sel_ids;     // int32  [n_slots][sel_cap]
  size_t tok_list;    // int32  [n_slots][list_cap]
  size_t err;         // int32  [4]
  size_t idx_mask;    // uint32 [n_slots][IDX_MASK_WORDS]  index tokens of the chunk appended last (dynamic index vectors)
  // host-offloaded KV only (else row_list == tok_list and the pools are empty):
  size_t row_list;    // int32  [n_slots][list_cap]  the context list as rows of the device pool
  size_t k_pool;      // dtype  [n_slots][pool_rows][d]  initial tokens | ring of the latest tokens | retrieved rows
  size_t v_pool;      // dtype  [n_slots][pool_rows][d]
  size_t total;
};

// Byte offsets inside `scratch` for one batch of segmentation problems.
struct ScratchLayout {
  size_t rowsum;   // double [P][nb][Lp]   tile row sums, indexed [J][i]
  size_t csuf;     // double [P][nb][Lp]   suffix-scanned tile column sums, indexed [I][x]
  size_t tsum;     // double [P][nb][nb]
  size_t rcar;     // double [P][nb][Lp]   row carry  RC[J][i]
  size_t ccar;     // double [P][nb][Lp]   column carry A[I][x]
  size_t pscore;   // double [P][ntiles][128]
  size_t px;       // int32  [P][ntiles][128]
  size_t ckey;     // uint64 [P][SEG_MAX_DIAG]  merged candidates: order key per anti-diagonal
  size_t cxy;      // uint32 [P][SEG_MAX_DIAG]  x << 16 | y
  size_t lse;      // double [P][G][Lp]    (SOFTMAX map only)
  size_t qrep;     // dtype  [n_seqs * Hkv][Lp][d]
  size_t qpart;    // double [2][P][Lp / 128 + Lp][d]  sums of 128-token pieces of query spans, or running sums of the
                   //        chunk's query rows [0] and key rows [1]
  size_t bounds;   // int32  [Hkv][chunk_max + 1] + int32 [Hkv]  (append_with_spans)
  size_t selflag;  // uint8  [n_seqs * Hkv][max_spans]  1 = span selected (between the two selection kernels)
  size_t att_part; // float  [n_seqs][Hq][ATT_MAX_SPLITS][ATT_SPLIT_MAX_ROWS][d + 2]  partial attention results
  size_t tokspan;  // int32  [P][Lp]      span (within the chunk) of every token (dynamic index vectors)
  size_t dyn;      // double [P][3][Lp]   votes, in-span row sums, whole row sums of the softmax map
  size_t qhist;    // uint32 [P][QUANT_BINS]  histogram of one digit of the map cells' order keys (percentile theta)
  size_t qstate;   // uint64 [P][QUANT_STATE_WORDS]   key prefix found so far, rank still to go, theta (double bits), status, list length
  size_t qlist;    // uint64 [P][QUANT_LISTS][QUANT_LIST_CAP]  order keys of the cells that share the prefix (percentile theta only)
  size_t lpart;    // double [P][G][nb][Lp][2]  per tile: row maximum and sum of exponentials (row log-sum-exp in pieces)
  size_t att_lse2; // float  [n_seqs][chunk_max][Hq]  log-sum-exp of the first part of a two-part step
  size_t loclist;  // int32  [n_seqs][loc_cap]  initial | window tokens (two-part step)
  size_t tickets;  // int32  [2][P]  finished workgroups per problem (step 2 of long chunks); zero between launches
  size_t total;
  int    loc_cap;       // entries of one sequence's initial | window list, whole tiles plus one
  int    max_problems;  // P the buffer was sized for
};

struct Dims {
  int Hq, Hkv, G, d, dtype, n_layers, n_seqs;
  long long max_tokens;
  int chunk_max, n_sink, window, k_max;
  long long budget;
  int seg_map;
  float theta, phi;
  int max_keep;
  int max_spans, sel_cap, list_cap;
  int elt;  // bytes per element
  int rep_mode, index_min, index_max, ratio_mode;   // dynamic index vectors (Sec. 3.3.2)
  int index_block_max;                              // > 0: at most this many index vectors per memory block, shared over its spans
  double lambda;
  double theta_quantile;                            // > 0: theta is this percentile of the chunk's map
  int unit;                                         // > 0: retrieval by memory units of this many tokens (Eq. 9)
  // Where the kernels find K/V rows. Resident KV: a slot's rows are its tokens, arena_rows = max_tokens, and
  // ring_mask = -1, ring0 = stage0 = 0. Host-offloaded KV (Sec. 3.4 first step: evicted tokens live in CPU
  // memory): a slot's rows on the device are a pool of arena_rows rows = the initial tokens [0, n_sink) | a
  // ring of ring_mask + 1 rows plus chunk_max mirror rows from ring0 (token t at ring0 + (t & ring_mask); a
  // chunk is written without a break, its part past the ring's end again at the ring's start) | the rows
  // fetched for the retrieved tokens from stage0 on.
  int offload;
  long long arena_rows;
  int ring0, ring_mask, stage0;
};

struct BatchPos {            // per-sequence values of one batched call
  int32_t seq[LTRI_MAX_BATCH];
  int32_t c0[LTRI_MAX_BATCH];   // chunk start (tokens already in the stream)
};

// Voters of a collaborative retrieval (Sec. 3.5): earlier layers and their weights, then the layer's own weight.
constexpr int VOTE_MAX_LAYERS = 64;
constexpr int VOTE_MAX_UNITS = 4096;     // units of a full stream the voting kernel holds in LDS
struct VoteArgs {
  int n_voters;
  int layer[VOTE_MAX_LAYERS];
  float weight[VOTE_MAX_LAYERS];
  float own_weight;
};

// Raw device views handed to the kernels.
struct DevState {
  int32_t* meta; int32_t* span_start; int32_t* span_len; void* krep; double* scores;
  int32_t* sel_ids; int32_t* tok_list; int32_t* err; uint32_t* idx_mask;
  int32_t* row_list;       // what the attention walks: tok_list itself, or (host-offloaded KV) the same list as pool rows
};
struct DevScratch {
  double* rowsum; double* csuf; double* tsum; double* rcar; double* ccar;
  double* pscore; int32_t* px; uint64_t* ckey; uint32_t* cxy; double* lse; void* qrep; double* qpart; int32_t* bounds; uint8_t* selflag; float* att_part;
  int32_t* tokspan; double* dyn; double* lpart; uint32_t* qhist; unsigned long long* qstate;
  float* att_lse2; int32_t* loclist;
  unsigned long long* qlist;
  int32_t* tickets;   // [2][max_problems] counters of finished workgroups; zero between launches
};

// Running sums of a chunk's query and key rows (running_sums.h), which step 2 of long chunks with mean
// representatives reads instead of summing the rows of every span.
struct RunSums {
  const void* q;         // [seq][n_q][Hq][128] query rows of the chunk
  const void* k_arena;   // key rows (the chunk's are in place), or NULL: no running sums of keys
  double* out;           // [problem][rows][128]
  size_t keys_off;       // elements from the query rows' sums to the key rows'
  int n_q;
  int rows;              // rows per problem in `out`
};
// Whether step 2 of a chunk of n_q tokens can read running sums (launch_retrieve decides with the span count at hand).
bool retrieve_reads_running_sums(const Dims& D, int n_q);
// Where they go: the buffer of the query-span pieces, which such a step does not use.
inline RunSums running_sums_of(const Dims& D, const DevScratch& sc, int sc_max_problems, const void* q,
                               const void* k_arena, int n_q) {
  RunSums r;
  r.q = q; r.k_arena = k_arena; r.out = sc.qpart; r.n_q = n_q;
  r.rows = n_q / 128 + n_q;
  r.keys_off = (size_t)sc_max_problems * r.rows * D.d;
  return r;
}

// ---- launchers (each returns the hipError_t of the launch) ----
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t launch_copy_chunk(const Dims& D, void* k_arena, void* v_arena, const void* k_chunk,
                             const void* v_chunk, int layer, const BatchPos& bp, int seq_count,
                             int n_new, void* k_host, void* v_host, hipStream_t s);   // k_host / v_host: the host arenas of an offloaded context, else NULL
// host-offloaded KV: rows of the retrieved tokens of the current list, host arenas -> device pool
hipError_t launch_fetch_retrieved(const Dims& D, const DevState& st, void* k_pool, void* v_pool, const void* k_host,
                                  const void* v_host, int layer, const BatchPos& bp, int seq_count, hipStream_t s);
hipError_t launch_segment(const Dims& D, const DevState& st, const DevScratch& sc, const void* k_arena,
                          const void* q_seg, int layer, const BatchPos& bp, int batch_off, int seq_count,
                          int n_new, hipEvent_t after_tiles, const RunSums* sums, hipStream_t s);
// event (or NULL): recorded behind the last kernel that fills the chip; sums (or NULL): further workgroups of the
// first tile launch take these running sums
hipError_t launch_append_single(const Dims& D, const DevState& st, const void* k_arena, int layer,
                                const BatchPos& bp, int seq_count, hipStream_t s);
hipError_t launch_append_bounds(const Dims& D, const DevState& st, const DevScratch& sc, int layer,
                                int seq, int c0, int n_new, hipStream_t s);
hipError_t launch_dynamic_reps(const Dims& D, const DevState& st, const DevScratch& sc, const void* k_arena,
                               const void* q_seg, int layer, const BatchPos& bp, int batch_off, int seq_count,
                               int n_new, bool lse_ready, hipEvent_t after_tiles, hipStream_t s);   // event as in launch_segment
hipError_t launch_rep_keys(const Dims& D, const DevState& st, const void* k_arena, int layer,
                           const BatchPos& bp, int seq_count, int n_new, hipStream_t s);
hipError_t launch_retrieve(const Dims& D, const DevState& st, const DevScratch& sc, int sc_max_problems,
                           const void* q, int layer, const BatchPos& bp, int seq_count, int n_q, int span_bound,
                           int32_t* sel_ids_out, int32_t* sel_cnt_out, const VoteArgs* votes, const void* append_k_arena,
                           const void* rep_k_arena, bool sums_ready, hipStream_t s);
// append_k_arena (or NULL): a one-token chunk's step 1 runs in the same launch; rep_k_arena (or NULL): the step
// also stores the chunk's mean keys (only where retrieve_stores_rep_keys says so); sums_ready: the running sums of
// running_sums_of(D, sc, sc_max_problems, q, rep_k_arena, n_q) are in place (one batch of sequences only)
bool retrieve_stores_rep_keys(const Dims& D, int n_q);
bool retrieve_is_one_launch(const Dims& D, int n_q, int span_bound);   // step 2 of a one-token chunk as a single kernel
hipError_t launch_persist_list(const Dims& D, const DevState& st, int layer, const BatchPos& bp, int seq_count,
                               hipStream_t s);
hipError_t launch_force_list(const Dims& D, const DevState& st, int layer, int seq, int kv_head,
                             int n_ids, hipStream_t s);
hipError_t launch_attend(const Dims& D, const DevState& st, const void* k_arena, const void* v_arena,
                         const void* q, int layer, const BatchPos& bp, int seq_count, int n_q,
                         void* out, float* lse, int stages, float* part, int part_mode, const int32_t* loclist,
                         int loc_cap, const float* lse_a,
                         hipStream_t s, hipEvent_t t_begin = nullptr, hipEvent_t t_end = nullptr);
// lse_a: the first part's log-sum-exp, for the retrieved part. t_begin / t_end (both or neither): timing events. The
// matrix-core kernel carries them in its own dispatch (they take the kernel's start and end time stamps, and no
// marker is queued that the neighbouring launches would wait behind); other shapes record them around the launches.
// bytes of partial results a launch over seq_count sequences with n_q query rows needs (0: the key range is not split)
size_t attend_partial_bytes(const Dims& D, int seq_count, int n_q, int n_cus);
// device address, on the current device, of the library's own buffer of ATT_STATIC_SCRATCH_BYTES for partial results
hipError_t attend_static_scratch(float** ptr);
bool attend_on_matrix_cores(const Dims& D);      // the bf16 kernel takes this shape (else one wavefront per query row)
hipError_t launch_local_list(const Dims& D, const BatchPos& bp, int seq_count, int32_t* loclist, int loc_cap,
                             hipStream_t s);
hipError_t launch_gather_pack(const Dims& D, const DevState& st, const void* k_arena, const void* v_arena,
                              int layer, int seq, void* k_packed, void* v_packed, int32_t* n_tokens,
                              hipStream_t s);

}  // namespace ltri
