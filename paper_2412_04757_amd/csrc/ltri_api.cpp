// Host side of libltri: context, argument checks, buffer layout, kernel sequencing.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "ltri_internal.h"

using namespace ltri;

struct ltri_ctx {
  ltri_config cfg;
  Dims D;
  StateLayout SL;
  ScratchLayout CL;
  char* k_arena; char* v_arena; char* state; char* scratch;   // k_arena / v_arena: where the kernels read K/V rows (offloaded KV: the device pools inside `state`)
  char* k_host; char* v_host;                                  // offloaded KV: the caller's host arenas, else NULL
  hipStream_t stream;
  DevState ds;
  DevScratch dc;
  bool dry;
  int attend_stages;                     // LDS ring depth of the bf16 attention kernel (3 or 4)
  int step_stages;                       // the same for the two parts of a step with host-offloaded keys and values
  // second stream and the fork / join events of such a step
  hipStream_t side; hipEvent_t ev_fork, ev_join;
  int n_cus;                             // compute units of the device
  float* static_part;                    // the library's own buffer for partial attention results on this context's device
  // optional timing of the attention launches of ltri_step: four events per step (around the one launch and an
  // empty interval, or around the first part on the second stream and the retrieved part on the context's
  // stream), reused after every read
  bool step_timing;
  std::vector<hipEvent_t> tev;
  size_t tev_used;
  std::vector<uint8_t> tev_parts;     // events of each recorded step: 2 (one attention launch) or 4 (two)
  // host mirror of the stream positions, per (layer, seq)
  std::vector<long long> n_tokens;       // tokens appended
  std::vector<int> last_len;             // length of the chunk appended last (0 = none)
  std::vector<long long> span_bound;     // upper bound on the spans stored per KV head
  std::vector<uint32_t> have_sel;        // bit h set: KV head h has a selection for the last chunk
  std::vector<uint32_t> ever_sel;        // bit h set: KV head h has had a selection since the last reset
  // sequences whose percentile threshold the device still holds (the last segmentation launch): layer, first, count
  int theta_layer = -1, theta_seq0 = 0, theta_seqs = 0;
  std::string err;
};

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int32_t fail(ltri_ctx* c, int32_t code, const char* fmt, ...) {
  if (c) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    c->err = buf;
  }
  return code;
}

static int32_t derive(const ltri_config* cfg, Dims& D, StateLayout& SL, ScratchLayout& CL) {
  if (!cfg) return LTRI_EINVAL;
  const ltri_config& c = *cfg;
  if (c.n_q_heads < 1 || c.n_kv_heads < 1 || c.n_q_heads % c.n_kv_heads) return LTRI_EINVAL;
  if (c.dtype != LTRI_F32 && c.dtype != LTRI_BF16) return LTRI_EINVAL;
  if (c.head_dim != 64 && c.head_dim != 128) return LTRI_EINVAL;
  if (c.dtype == LTRI_BF16 && c.head_dim != 128) return LTRI_EINVAL;
  // the bf16 attention kernel addresses a KV head's rows with 32-bit byte offsets
  if (c.dtype == LTRI_BF16 && c.max_tokens >= (1ll << 24)) return LTRI_EINVAL;
  if (c.n_layers < 1 || c.n_seqs < 1 || c.max_tokens < 1 || c.max_tokens > (1ll << 30)) return LTRI_EINVAL;
  if (c.chunk_max < 1 || c.chunk_max > SEG_MAX_L) return LTRI_EINVAL;
  if (c.n_sink < 0 || c.window < 0 || c.k_max < 0 || c.budget_tokens < 0) return LTRI_EINVAL;
  if (c.seg_map != LTRI_MAP_SOFTMAX && c.seg_map != LTRI_MAP_LOGIT) return LTRI_EINVAL;
  if (!(c.phi >= 0.0f) || !(c.theta == c.theta)) return LTRI_EINVAL;
  if (c.max_spans_per_chunk < 0 || c.max_spans < 0) return LTRI_EINVAL;
  if (c.rep_mode != LTRI_REP_MEAN && c.rep_mode != LTRI_REP_DYNAMIC) return LTRI_EINVAL;
  if (!(c.theta_quantile >= 0.0f) || c.theta_quantile > 1.0f) return LTRI_EINVAL;
  if (c.unit_tokens < 0 || c.unit_tokens > c.chunk_max) return LTRI_EINVAL;
  if (c.unit_tokens > 0 && c.max_tokens / c.unit_tokens + 1 > 8192) return LTRI_EINVAL;
  if (c.rep_mode == LTRI_REP_DYNAMIC &&
      (!(c.lambda >= 0.0f) || c.index_min < 0 || c.index_max < 0 || (c.index_max && c.index_max < c.index_min) ||
       c.ratio_mode < LTRI_RATIO_ROW || c.ratio_mode > LTRI_RATIO_ROWCOL))
    return LTRI_EINVAL;
  const int G = c.n_q_heads / c.n_kv_heads;
  if (c.dtype == LTRI_BF16 && !(G == 1 || G == 2 || G % 4 == 0)) return LTRI_EINVAL;
  D.Hq = c.n_q_heads; D.Hkv = c.n_kv_heads; D.G = G; D.d = c.head_dim; D.dtype = c.dtype;
  D.n_layers = c.n_layers; D.n_seqs = c.n_seqs; D.max_tokens = c.max_tokens;
  D.chunk_max = c.chunk_max; D.n_sink = c.n_sink; D.window = c.window; D.k_max = c.k_max;
  D.budget = c.budget_tokens; D.seg_map = c.seg_map; D.theta = c.theta; D.phi = c.phi;
  D.max_keep = c.max_spans_per_chunk;
  D.rep_mode = c.rep_mode; D.lambda = (double)c.lambda; D.index_min = c.index_min; D.index_max = c.index_max;
  D.ratio_mode = c.ratio_mode;
  D.theta_quantile = (double)c.theta_quantile;
  D.unit = c.unit_tokens;
  if (c.index_block_max < 0) return LTRI_EINVAL;
  if (c.index_block_max > 0 && (c.rep_mode != LTRI_REP_DYNAMIC || c.unit_tokens <= 0)) return LTRI_EINVAL;
  D.index_block_max = c.index_block_max;
  if (c.kv_offload != 0 && c.kv_offload != 1) return LTRI_EINVAL;
  D.offload = c.kv_offload;
  if (c.max_spans > 65536) return LTRI_EINVAL;
  long long ms = c.max_spans ? c.max_spans : std::min<long long>(c.max_tokens / 32 + 64, 65536);
  if (ms > c.max_tokens) ms = c.max_tokens;
  if (ms < 1 || ms > 65536) return LTRI_EINVAL;
  D.max_spans = (int)ms;
  long long sel = ms;
  if (c.k_max) sel = std::min<long long>(sel, c.k_max);
  if (c.budget_tokens) sel = std::min<long long>(sel, c.budget_tokens);
  D.sel_cap = (int)std::max<long long>(sel, 1);
  long long ret = c.max_tokens;
  if (c.budget_tokens) ret = std::min<long long>(ret, c.budget_tokens);
  if (c.k_max) ret = std::min<long long>(ret, (long long)c.k_max * c.chunk_max);
  long long lc = std::min<long long>(c.max_tokens, (long long)c.n_sink + ret + c.window);
  lc = (long long)align_up((size_t)lc, ATT_BN) + ATT_BN;
  if (lc > (1ll << 30)) return LTRI_EINVAL;
  D.list_cap = (int)lc;
  D.elt = c.dtype == LTRI_F32 ? 4 : 2;
  if (D.offload) {
    // device pool of a slot: initial tokens | ring (a power of two of at least window + 2 chunks, so that the next
    // chunk can be appended while the last one is still attended) + one chunk of mirror rows | retrieved rows
    long long ring = 64;
    while (ring < (long long)c.window + 2ll * c.chunk_max) ring <<= 1;
    if (ring > (1ll << 24)) return LTRI_EINVAL;
    D.ring0 = c.n_sink;
    D.ring_mask = (int)(ring - 1);
    D.stage0 = (int)(c.n_sink + ring + c.chunk_max);
    D.arena_rows = (long long)D.stage0 + D.list_cap;
  } else {
    D.ring0 = 0; D.ring_mask = -1; D.stage0 = 0;
    D.arena_rows = c.max_tokens;
  }

  const size_t n_slots = (size_t)c.n_layers * c.n_seqs * c.n_kv_heads;
  size_t o = 0;
  SL.meta = o;       o = align_up(o + n_slots * META_WORDS * 4, 256);
  SL.span_start = o; o = align_up(o + n_slots * D.max_spans * 4, 256);
  SL.span_len = o;   o = align_up(o + n_slots * D.max_spans * 4, 256);
  SL.krep = o;       o = align_up(o + n_slots * D.max_spans * (size_t)D.d * D.elt, 256);
  SL.scores = o;     o = align_up(o + n_slots * D.max_spans * 8, 256);
  SL.sel_ids = o;    o = align_up(o + n_slots * D.sel_cap * 4, 256);
  SL.tok_list = o;   o = align_up(o + n_slots * (size_t)D.list_cap * 4, 256);
  SL.err = o;        o = align_up(o + 16, 256);
  SL.idx_mask = o;   o = align_up(o + n_slots * IDX_MASK_WORDS * 4, 256);
  SL.row_list = o;   o = align_up(o + (D.offload ? n_slots * (size_t)D.list_cap * 4 : 0), 256);
  SL.k_pool = o;     o = align_up(o + (D.offload ? n_slots * (size_t)D.arena_rows * D.d * D.elt : 0), 256);
  SL.v_pool = o;     o = align_up(o + (D.offload ? n_slots * (size_t)D.arena_rows * D.d * D.elt : 0), 256);
  SL.total = o;

  // scratch: segmentation temporaries for up to 4 sequences at a time
  const int P = std::min(c.n_seqs, 4) * c.n_kv_heads;
  const size_t nb = (c.chunk_max + SEG_TB - 1) / SEG_TB, Lp = nb * SEG_TB, nt = nb * (nb + 1) / 2;
  o = 0;
  CL.rowsum = o; o = align_up(o + (size_t)P * nb * Lp * 8, 256);
  CL.csuf = o;   o = align_up(o + (size_t)P * nb * Lp * 8, 256);
  CL.tsum = o;   o = align_up(o + (size_t)P * nb * nb * 8, 256);
  CL.rcar = o;   o = align_up(o + (size_t)P * nb * Lp * 8, 256);
  CL.ccar = o;   o = align_up(o + (size_t)P * nb * Lp * 8, 256);
  CL.pscore = o; o = align_up(o + (size_t)P * nt * 128 * 8, 256);
  CL.px = o;     o = align_up(o + (size_t)P * nt * 128 * 4, 256);
  CL.ckey = o;   o = align_up(o + (size_t)P * SEG_MAX_DIAG * 8, 256);
  CL.cxy = o;    o = align_up(o + (size_t)P * SEG_MAX_DIAG * 4, 256);
  CL.lse = o;    o = align_up(o + (size_t)P * G * Lp * 8, 256);
  // query-span representatives are needed for every sequence of a batched retrieve
  CL.qrep = o;   o = align_up(o + (size_t)c.n_seqs * c.n_kv_heads * Lp * D.d * D.elt, 256);
  CL.qpart = o;  o = align_up(o + (size_t)2 * P * (Lp / 128 + Lp) * D.d * 8, 256);
  CL.bounds = o; o = align_up(o + (size_t)c.n_kv_heads * (c.chunk_max + 2) * 4, 256);
  CL.selflag = o; o = align_up(o + (size_t)c.n_seqs * c.n_kv_heads * D.max_spans, 256);
  CL.att_part = o; o = align_up(o + (size_t)c.n_seqs * c.n_q_heads * ATT_MAX_SPLITS * ATT_SPLIT_MAX_ROWS * (D.d + 2) * 4, 256);
  CL.tokspan = o; o = align_up(o + (size_t)P * Lp * 4, 256);
  CL.dyn = o;     o = align_up(o + (size_t)P * 3 * Lp * 8, 256);
  CL.qhist = o;   o = align_up(o + (size_t)P * QUANT_BINS * 4, 256);
  CL.qstate = o;  o = align_up(o + (size_t)P * QUANT_STATE_WORDS * 8, 256);
  CL.qlist = o;   o = align_up(o + (c.theta_quantile > 0.0 ? (size_t)P * QUANT_LISTS * QUANT_LIST_CAP * 8 : 0), 256);
  CL.lpart = o;   o = align_up(o + (c.rep_mode == LTRI_REP_DYNAMIC || c.seg_map == LTRI_MAP_SOFTMAX ? (size_t)P * G * nb * Lp * 16 : 0), 256);
  CL.loc_cap = (int)align_up((size_t)c.n_sink + c.window, ATT_BN) + ATT_BN;
  CL.att_lse2 = o;  o = align_up(o + (size_t)c.n_seqs * c.chunk_max * c.n_q_heads * 4, 256);
  CL.loclist = o;   o = align_up(o + (size_t)c.n_seqs * CL.loc_cap * 4, 256);
  CL.tickets = o;   o = align_up(o + (size_t)2 * P * 4, 256);
  CL.total = o;
  CL.max_problems = P;
  return LTRI_OK;
}

extern "C" {

const char* ltri_version(void) { return "libltri 0.1 gfx950"; }

const char* ltri_strerror(int32_t s) {
  switch (s) {
    case LTRI_OK: return "ok";
    case LTRI_EINVAL: return "invalid argument or unsupported configuration";
    case LTRI_ESTATE: return "call out of order";
    case LTRI_ECAPACITY: return "token or span capacity exceeded";
    case LTRI_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* ltri_last_error(const ltri_ctx* c) { return c ? c->err.c_str() : ""; }

int32_t ltri_workspace_bytes(const ltri_config* cfg, size_t* state_bytes, size_t* scratch_bytes) {
  Dims D; StateLayout SL; ScratchLayout CL;
  const int32_t r = derive(cfg, D, SL, CL);
  if (r != LTRI_OK) return r;
  if (state_bytes) *state_bytes = SL.total;
  if (scratch_bytes) *scratch_bytes = CL.total;
  return LTRI_OK;
}

static int32_t create_impl(const ltri_config* cfg, void* k_arena, void* v_arena, void* state, void* scratch,
                           void* hip_stream, bool dry, ltri_ctx** out) {
  if (!out) return LTRI_EINVAL;
  *out = nullptr;
  Dims D; StateLayout SL; ScratchLayout CL;
  const int32_t r = derive(cfg, D, SL, CL);
  if (r != LTRI_OK) return r;
  if (!dry) {
    if (!k_arena || !v_arena || !state || !scratch) return LTRI_EINVAL;
    if (((uintptr_t)k_arena | (uintptr_t)v_arena | (uintptr_t)state | (uintptr_t)scratch) & 255) return LTRI_EINVAL;
  }
  ltri_ctx* c = new (std::nothrow) ltri_ctx();
  if (!c) return LTRI_EINVAL;
  c->cfg = *cfg; c->D = D; c->SL = SL; c->CL = CL;
  c->state = (char*)state; c->scratch = (char*)scratch;
  if (D.offload && !dry) {
    // the host arenas must be pinned memory the device can address: the kernels use the device's view of them
    void* dev_view[2] = {nullptr, nullptr};
    void* given[2] = {k_arena, v_arena};
    for (int i = 0; i < 2; ++i) {
      hipPointerAttribute_t at;
      memset(&at, 0, sizeof at);
      const hipError_t e = hipPointerGetAttributes(&at, given[i]);
      if (e != hipSuccess || at.type != hipMemoryTypeHost || !at.devicePointer) {
        (void)hipGetLastError();
        delete c;
        return LTRI_EINVAL;
      }
      dev_view[i] = at.devicePointer;
    }
    c->k_host = (char*)dev_view[0]; c->v_host = (char*)dev_view[1];
    c->k_arena = c->state + SL.k_pool; c->v_arena = c->state + SL.v_pool;
  } else {
    c->k_host = nullptr; c->v_host = nullptr;
    c->k_arena = (char*)k_arena; c->v_arena = (char*)v_arena;
  }
  c->stream = (hipStream_t)hip_stream;
  c->dry = dry;
  c->attend_stages = 4;
  c->step_stages = 4;
  c->side = nullptr; c->ev_fork = nullptr; c->ev_join = nullptr;
  c->n_cus = 0;
  c->static_part = nullptr;
  c->step_timing = false; c->tev_used = 0;
  char* s = c->state;
  c->ds = DevState{(int32_t*)(s + SL.meta), (int32_t*)(s + SL.span_start), (int32_t*)(s + SL.span_len),
                   (void*)(s + SL.krep), (double*)(s + SL.scores), (int32_t*)(s + SL.sel_ids),
                   (int32_t*)(s + SL.tok_list), (int32_t*)(s + SL.err), (uint32_t*)(s + SL.idx_mask),
                   (int32_t*)(s + (D.offload ? SL.row_list : SL.tok_list))};
  char* t = c->scratch;
  c->dc = DevScratch{(double*)(t + CL.rowsum), (double*)(t + CL.csuf), (double*)(t + CL.tsum),
                     (double*)(t + CL.rcar), (double*)(t + CL.ccar), (double*)(t + CL.pscore),
                     (int32_t*)(t + CL.px), (uint64_t*)(t + CL.ckey), (uint32_t*)(t + CL.cxy), (double*)(t + CL.lse), (void*)(t + CL.qrep),
                     (double*)(t + CL.qpart), (int32_t*)(t + CL.bounds), (uint8_t*)(t + CL.selflag), (float*)(t + CL.att_part),
                     (int32_t*)(t + CL.tokspan), (double*)(t + CL.dyn), (double*)(t + CL.lpart),
                     (uint32_t*)(t + CL.qhist), (unsigned long long*)(t + CL.qstate),
                     (float*)(t + CL.att_lse2), (int32_t*)(t + CL.loclist), (unsigned long long*)(t + CL.qlist),
                     (int32_t*)(t + CL.tickets)};
  const size_t n = (size_t)D.n_layers * D.n_seqs;
  c->n_tokens.assign(n, 0);
  c->last_len.assign(n, 0);
  c->span_bound.assign(n, 0);
  c->have_sel.assign(n, 0u);
  c->ever_sel.assign(n, 0u);
  if (!dry) {
    hipError_t e = launch_fill_zero(c->state, SL.total, c->stream);
    if (e == hipSuccess) e = launch_fill_zero(c->scratch + CL.tickets, align_up((size_t)2 * CL.max_problems * 4, 256), c->stream);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
    // the two events order streams of this device only: no timing, and a device-scope release when they are recorded
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming | hipEventReleaseToDevice);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming | hipEventReleaseToDevice);
    int dev = 0;
    if (e == hipSuccess) e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = attend_static_scratch(&c->static_part);   // set-up: the device address of the library's own buffer
    if (e != hipSuccess) { ltri_destroy(c); return LTRI_EHIP; }
  }
  *out = c;
  return LTRI_OK;
}

int32_t ltri_create(const ltri_config* cfg, void* k_arena, void* v_arena, void* state, void* scratch,
                    void* hip_stream, ltri_ctx** out) {
  return create_impl(cfg, k_arena, v_arena, state, scratch, hip_stream, false, out);
}

int32_t ltri_create_dry(const ltri_config* cfg, ltri_ctx** out) {
  return create_impl(cfg, nullptr, nullptr, nullptr, nullptr, nullptr, true, out);
}

int32_t ltri_destroy(ltri_ctx* c) {
  if (!c) return LTRI_EINVAL;
  if (c->side) {      // work of a two-part step may still be queued there
    (void)hipStreamSynchronize(c->side);
    (void)hipStreamDestroy(c->side);
  }
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  if (c->ev_join) (void)hipEventDestroy(c->ev_join);
  for (hipEvent_t e : c->tev) (void)hipEventDestroy(e);
  delete c;
  return LTRI_OK;
}

int32_t ltri_set_stream(ltri_ctx* c, void* hip_stream) {
  if (!c) return LTRI_EINVAL;
  c->stream = (hipStream_t)hip_stream;
  return LTRI_OK;
}

int32_t ltri_set_attend_stages(ltri_ctx* c, int32_t stages) {
  if (!c) return LTRI_EINVAL;
  if (stages != 3 && stages != 4) return fail(c, LTRI_EINVAL, "attend stages must be 3 or 4");
  c->attend_stages = stages;
  c->step_stages = stages;
  return LTRI_OK;
}

int32_t ltri_sel_capacity(const ltri_ctx* c) { return c ? c->D.sel_cap : LTRI_EINVAL; }
int32_t ltri_list_capacity(const ltri_ctx* c) { return c ? c->D.list_cap : LTRI_EINVAL; }

}  // extern "C"

// ------------------------------------------------------------------------------------------
static int32_t check_hip(ltri_ctx* c, hipError_t e, const char* what) {
  if (e == hipSuccess) return LTRI_OK;
  return fail(c, LTRI_EHIP, "%s: %s", what, hipGetErrorString(e));
}

static int32_t check_range(ltri_ctx* c, int layer, int seq_begin, int seq_count) {
  if (!c) return LTRI_EINVAL;
  if (layer < 0 || layer >= c->D.n_layers) return fail(c, LTRI_EINVAL, "layer %d out of range", layer);
  if (seq_count < 1 || seq_count > LTRI_MAX_BATCH || seq_begin < 0 || seq_begin + seq_count > c->D.n_seqs)
    return fail(c, LTRI_EINVAL, "sequence range [%d, %d) invalid", seq_begin, seq_begin + seq_count);
  return LTRI_OK;
}

static size_t ls_index(const ltri_ctx* c, int layer, int seq) { return (size_t)layer * c->D.n_seqs + seq; }

// Host-offloaded KV: once a selection's token list is written, the rows of its retrieved tokens are fetched from
// the host arenas into the device pool, on the context's stream, before anything attends.
static int32_t fetch_retrieved(ltri_ctx* c, int layer, const BatchPos& bp, int seq_count, hipStream_t s = nullptr) {
  if (!c->D.offload || c->dry) return LTRI_OK;
  return check_hip(c, launch_fetch_retrieved(c->D, c->ds, c->k_arena, c->v_arena, c->k_host, c->v_host, layer, bp,
                                             seq_count, s ? s : c->stream), "fetch retrieved rows");
}

extern "C" {

int32_t ltri_reset(ltri_ctx* c, int32_t seq) {
  if (!c) return LTRI_EINVAL;
  if (seq < 0 || seq >= c->D.n_seqs) return fail(c, LTRI_EINVAL, "sequence %d out of range", seq);
  for (int l = 0; l < c->D.n_layers; ++l) {
    const size_t i = ls_index(c, l, seq);
    c->n_tokens[i] = 0; c->last_len[i] = 0; c->span_bound[i] = 0; c->have_sel[i] = 0; c->ever_sel[i] = 0;
    if (!c->dry) {
      const size_t off = c->SL.meta + ((size_t)(l * c->D.n_seqs + seq) * c->D.Hkv) * META_WORDS * 4;
      // META_WORDS * 4 = 32 bytes per slot: the slots of one (layer, seq) are contiguous
      const int32_t r = check_hip(c, launch_fill_zero(c->state + off, (size_t)c->D.Hkv * META_WORDS * 4, c->stream),
                                  "reset");
      if (r != LTRI_OK) return r;
    }
  }
  return LTRI_OK;
}

static int32_t append_common(ltri_ctx* c, int layer, int seq_begin, int seq_count, const void* k_chunk,
                             const void* v_chunk, int n_new, BatchPos& bp) {
  int32_t r = check_range(c, layer, seq_begin, seq_count);
  if (r != LTRI_OK) return r;
  if (n_new < 1 || n_new > c->D.chunk_max)
    return fail(c, LTRI_EINVAL, "n_new %d outside [1, chunk_max %d]", n_new, c->D.chunk_max);
  if ((k_chunk == nullptr) != (v_chunk == nullptr))
    return fail(c, LTRI_EINVAL, "k_chunk and v_chunk must both be given or both be NULL");
  if (c->D.offload && !k_chunk)
    return fail(c, LTRI_EINVAL, "host-offloaded KV: the chunk's rows must be passed (k_chunk / v_chunk), the device holds no arena to find them in");
  for (int s = 0; s < seq_count; ++s) {
    const size_t i = ls_index(c, layer, seq_begin + s);
    if (c->n_tokens[i] + n_new > c->D.max_tokens)
      return fail(c, LTRI_ECAPACITY, "sequence %d: %lld + %d tokens exceed max_tokens %lld", seq_begin + s,
                  c->n_tokens[i], n_new, c->D.max_tokens);
    bp.seq[s] = seq_begin + s;
    bp.c0[s] = (int32_t)c->n_tokens[i];
  }
  if (k_chunk && !c->dry) {
    r = check_hip(c, launch_copy_chunk(c->D, c->k_arena, c->v_arena, k_chunk, v_chunk, layer, bp, seq_count,
                                       n_new, c->k_host, c->v_host, c->stream), "copy chunk");
    if (r != LTRI_OK) return r;
  }
  return LTRI_OK;
}

static void append_commit(ltri_ctx* c, int layer, int seq_begin, int seq_count, int n_new) {
  for (int s = 0; s < seq_count; ++s) {
    const size_t i = ls_index(c, layer, seq_begin + s);
    c->n_tokens[i] += n_new;
    c->last_len[i] = n_new;
    c->span_bound[i] = std::min<long long>(c->span_bound[i] + n_new, c->D.max_spans);
    c->have_sel[i] = 0;
  }
}

// Step 1 of a chunk whose rows are already in the arenas: segmentation and index vectors. `fork` (or NULL)
// is recorded on the context's stream behind the last kernel that fills the chip; what follows it there
// are kernels of a few workgroups each.
// q_step2 (or NULL): the query rows that step 2 will be called with right after; *sums_ready then says whether the
// running sums it reads were taken along by the segmentation's first launch.
static int32_t append_spans(ltri_ctx* c, int layer, const BatchPos& bp, int seq_count, const void* q_seg, int n_new,
                            hipEvent_t fork, bool rep_keys_later = false, const void* q_step2 = nullptr,
                            bool* sums_ready = nullptr) {
  int32_t r;
  if (sums_ready) *sums_ready = false;
  if (n_new == 1) {
    r = check_hip(c, launch_append_single(c->D, c->ds, c->k_arena, layer, bp, seq_count, c->stream),
                  "append (single token)");
    if (r == LTRI_OK && fork) r = check_hip(c, hipEventRecord(fork, c->stream), "fork");
    return r;
  }
  const int per = c->CL.max_problems / c->D.Hkv;     // sequences per segmentation launch
  const bool dynamic = c->D.rep_mode == LTRI_REP_DYNAMIC;
  // one batch of sequences only: the sums of a second batch would take the place of the first one's
  const bool with_sums = q_step2 && sums_ready && seq_count <= per && retrieve_reads_running_sums(c->D, n_new);
  RunSums sums;
  if (with_sums)
    sums = running_sums_of(c->D, c->dc, c->CL.max_problems, q_step2, rep_keys_later ? c->k_arena : nullptr, n_new);
  for (int off = 0; off < seq_count; off += per) {
    const int cnt = std::min(per, seq_count - off);
    const bool last = off + per >= seq_count;
    r = check_hip(c, launch_segment(c->D, c->ds, c->dc, c->k_arena, q_seg, layer, bp, off, cnt, n_new,
                                    last && !dynamic ? fork : nullptr, with_sums ? &sums : nullptr, c->stream), "segment");
    if (r != LTRI_OK) return r;
    if (dynamic) {
      r = check_hip(c, launch_dynamic_reps(c->D, c->ds, c->dc, c->k_arena, q_seg, layer, bp, off, cnt, n_new,
                                           c->D.seg_map == LTRI_MAP_SOFTMAX, last ? fork : nullptr, c->stream),
                    "index vectors");
      if (r != LTRI_OK) return r;
    }
    c->theta_layer = layer; c->theta_seq0 = bp.seq[off]; c->theta_seqs = cnt;
  }
  if (with_sums) *sums_ready = true;
  if (c->D.rep_mode == LTRI_REP_MEAN && !rep_keys_later) {   // later: step 2's first launch stores them as well
    r = check_hip(c, launch_rep_keys(c->D, c->ds, c->k_arena, layer, bp, seq_count, n_new, c->stream),
                  "representative keys");
    if (r != LTRI_OK) return r;
  }
  return LTRI_OK;
}

int32_t ltri_append_chunk(ltri_ctx* c, int32_t layer, int32_t seq_begin, int32_t seq_count,
                          const void* k_chunk, const void* v_chunk, const void* q_seg, int32_t n_new) {
  BatchPos bp;
  memset(&bp, 0, sizeof bp);
  int32_t r = append_common(c, layer, seq_begin, seq_count, k_chunk, v_chunk, n_new, bp);
  if (r != LTRI_OK) return r;
  if (!c->dry) {
    r = append_spans(c, layer, bp, seq_count, q_seg, n_new, nullptr);
    if (r != LTRI_OK) return r;
  }
  append_commit(c, layer, seq_begin, seq_count, n_new);
  return LTRI_OK;
}

int32_t ltri_append_chunk_with_spans(ltri_ctx* c, int32_t layer, int32_t seq, const void* k_chunk,
                                     const void* v_chunk, int32_t n_new, const int32_t* bounds_host,
                                     const int32_t* n_bounds_host) {
  BatchPos bp;
  memset(&bp, 0, sizeof bp);
  if (!c) return LTRI_EINVAL;
  if (!bounds_host || !n_bounds_host) return fail(c, LTRI_EINVAL, "bounds missing");
  // validate the boundaries before anything is enqueued
  if (n_new < 1 || n_new > c->D.chunk_max)
    return fail(c, LTRI_EINVAL, "n_new %d outside [1, chunk_max %d]", n_new, c->D.chunk_max);
  std::vector<int32_t> staged((size_t)c->D.Hkv * (c->D.chunk_max + 1) + c->D.Hkv, 0);
  size_t pos = 0;
  for (int h = 0; h < c->D.Hkv; ++h) {
    const int nbh = n_bounds_host[h];
    if (nbh < 2 || nbh > n_new + 1) return fail(c, LTRI_EINVAL, "head %d: %d boundaries", h, nbh);
    const int32_t* b = bounds_host + pos;
    if (b[0] != 0 || b[nbh - 1] != n_new) return fail(c, LTRI_EINVAL, "head %d: boundaries must run from 0 to n_new", h);
    for (int k = 1; k < nbh; ++k)
      if (b[k] <= b[k - 1]) return fail(c, LTRI_EINVAL, "head %d: boundaries not strictly increasing", h);
    memcpy(&staged[(size_t)h * (c->D.chunk_max + 1)], b, (size_t)nbh * 4);
    staged[(size_t)c->D.Hkv * (c->D.chunk_max + 1) + h] = nbh;
    pos += nbh;
  }
  int32_t r = append_common(c, layer, seq, 1, k_chunk, v_chunk, n_new, bp);
  if (r != LTRI_OK) return r;
  if (!c->dry) {
    r = check_hip(c, hipMemcpyAsync(c->dc.bounds, staged.data(), staged.size() * 4, hipMemcpyHostToDevice,
                                    c->stream), "copy boundaries");
    if (r != LTRI_OK) return r;
    r = check_hip(c, hipStreamSynchronize(c->stream), "copy boundaries (sync)");   // staged is a local
    if (r != LTRI_OK) return r;
    r = check_hip(c, launch_append_bounds(c->D, c->ds, c->dc, layer, seq, bp.c0[0], n_new, c->stream),
                  "append (given spans)");
    if (r != LTRI_OK) return r;
    if (c->D.rep_mode == LTRI_REP_DYNAMIC && n_new > 1)
      r = check_hip(c, launch_dynamic_reps(c->D, c->ds, c->dc, c->k_arena, nullptr, layer, bp, 0, 1, n_new, false,
                                           nullptr, c->stream), "index vectors");
    else
      r = check_hip(c, launch_rep_keys(c->D, c->ds, c->k_arena, layer, bp, 1, n_new, c->stream),
                    "representative keys");
    if (r != LTRI_OK) return r;
  }
  append_commit(c, layer, seq, 1, n_new);
  return LTRI_OK;
}

static int32_t check_query_chunk(ltri_ctx* c, int layer, int seq_begin, int seq_count, const void* q, int n_q,
                                 BatchPos& bp) {
  int32_t r = check_range(c, layer, seq_begin, seq_count);
  if (r != LTRI_OK) return r;
  if (!q) return fail(c, LTRI_EINVAL, "q is NULL");
  for (int s = 0; s < seq_count; ++s) {
    const size_t i = ls_index(c, layer, seq_begin + s);
    if (c->last_len[i] == 0) return fail(c, LTRI_ESTATE, "sequence %d: no chunk appended yet", seq_begin + s);
    if (c->last_len[i] != n_q)
      return fail(c, LTRI_ESTATE, "sequence %d: n_q %d differs from the last appended chunk (%d tokens)",
                  seq_begin + s, n_q, c->last_len[i]);
    bp.seq[s] = seq_begin + s;
    bp.c0[s] = (int32_t)(c->n_tokens[i] - n_q);
  }
  return LTRI_OK;
}

// fork and fetch_stream (both or neither; host-offloaded KV): the fetch of the retrieved rows is queued on that
// stream behind the event, which is recorded behind the kernels of step 2.
static int32_t retrieve_impl(ltri_ctx* c, int32_t layer, int32_t seq_begin, int32_t seq_count, const void* q,
                             int32_t n_q, int32_t* sel_ids, int32_t* sel_cnt, bool store_rep_keys,
                             bool sums_ready = false, hipEvent_t fork = nullptr, hipStream_t fetch_stream = nullptr) {
  BatchPos bp;
  memset(&bp, 0, sizeof bp);
  int32_t r = check_query_chunk(c, layer, seq_begin, seq_count, q, n_q, bp);
  if (r != LTRI_OK) return r;
  if (!c->dry) {
    long long bound = 0;
    for (int s = 0; s < seq_count; ++s) bound = std::max(bound, c->span_bound[ls_index(c, layer, seq_begin + s)]);
    r = check_hip(c, launch_retrieve(c->D, c->ds, c->dc, c->CL.max_problems, q, layer, bp, seq_count, n_q, (int)bound, sel_ids,
                                     sel_cnt, nullptr, nullptr, store_rep_keys ? c->k_arena : nullptr, sums_ready, c->stream),
                  "retrieve");
    if (r != LTRI_OK) return r;
    if (fork) {
      r = check_hip(c, hipEventRecord(fork, c->stream), "fork");
      if (r == LTRI_OK) r = check_hip(c, hipStreamWaitEvent(fetch_stream, fork, 0), "fork");
      if (r != LTRI_OK) return r;
    }
    r = fetch_retrieved(c, layer, bp, seq_count, fetch_stream);
    if (r != LTRI_OK) return r;
  }
  for (int s = 0; s < seq_count; ++s) {
    c->have_sel[ls_index(c, layer, seq_begin + s)] = 0xFFFFFFFFu;
    c->ever_sel[ls_index(c, layer, seq_begin + s)] = 0xFFFFFFFFu;
  }
  return LTRI_OK;
}

int32_t ltri_retrieve(ltri_ctx* c, int32_t layer, int32_t seq_begin, int32_t seq_count, const void* q,
                      int32_t n_q, int32_t* sel_ids, int32_t* sel_cnt) {
  return retrieve_impl(c, layer, seq_begin, seq_count, q, n_q, sel_ids, sel_cnt, false);
}

int32_t ltri_retrieve_collaborative(ltri_ctx* c, int32_t layer, int32_t seq_begin, int32_t seq_count, const void* q,
                                    int32_t n_q, const float* layer_weights_host, int32_t* sel_ids, int32_t* sel_cnt) {
  BatchPos bp;
  memset(&bp, 0, sizeof bp);
  int32_t r = check_query_chunk(c, layer, seq_begin, seq_count, q, n_q, bp);
  if (r != LTRI_OK) return r;
  if (c->D.unit <= 0) return fail(c, LTRI_EINVAL, "collaborative retrieval votes on memory units: unit_tokens is 0");
  if (!layer_weights_host) return fail(c, LTRI_EINVAL, "layer_weights_host is NULL");
  if (c->D.max_tokens / c->D.unit + 1 > VOTE_MAX_UNITS)
    return fail(c, LTRI_EINVAL, "collaborative retrieval holds at most %d units (max_tokens / unit_tokens + 1)", VOTE_MAX_UNITS);
  VoteArgs v;
  memset(&v, 0, sizeof v);
  const uint32_t need = c->D.Hkv >= 32 ? 0xFFFFFFFFu : ((1u << c->D.Hkv) - 1u);
  for (int l = 0; l <= layer; ++l) {
    const float w = layer_weights_host[l];
    if (!(w >= 0.0f)) return fail(c, LTRI_EINVAL, "weight of layer %d is negative or not a number", l);
    if (l == layer) { v.own_weight = w; break; }
    if (w == 0.0f) continue;
    if (v.n_voters == VOTE_MAX_LAYERS) return fail(c, LTRI_EINVAL, "more than %d voting layers", VOTE_MAX_LAYERS);
    for (int s = 0; s < seq_count; ++s) {
      const size_t iv = ls_index(c, l, seq_begin + s), io = ls_index(c, layer, seq_begin + s);
      if ((c->have_sel[iv] & need) != need || c->n_tokens[iv] != c->n_tokens[io] || c->last_len[iv] != c->last_len[io])
        return fail(c, LTRI_ESTATE, "layer %d has no selection for this chunk of sequence %d", l, seq_begin + s);
    }
    v.layer[v.n_voters] = l;
    v.weight[v.n_voters] = w;
    ++v.n_voters;
  }
  if (!c->dry) {
    long long bound = 0;
    for (int s = 0; s < seq_count; ++s) bound = std::max(bound, c->span_bound[ls_index(c, layer, seq_begin + s)]);
    r = check_hip(c, launch_retrieve(c->D, c->ds, c->dc, c->CL.max_problems, q, layer, bp, seq_count, n_q, (int)bound,
                                     sel_ids, sel_cnt, &v, nullptr, nullptr, false, c->stream), "collaborative retrieve");
    if (r != LTRI_OK) return r;
    r = fetch_retrieved(c, layer, bp, seq_count);
    if (r != LTRI_OK) return r;
  }
  for (int s = 0; s < seq_count; ++s) {
    c->have_sel[ls_index(c, layer, seq_begin + s)] = 0xFFFFFFFFu;
    c->ever_sel[ls_index(c, layer, seq_begin + s)] = 0xFFFFFFFFu;
  }
  return LTRI_OK;
}

int32_t ltri_retrieve_persistent(ltri_ctx* c, int32_t layer, int32_t seq_begin, int32_t seq_count) {
  int32_t r = check_range(c, layer, seq_begin, seq_count);
  if (r != LTRI_OK) return r;
  BatchPos bp;
  memset(&bp, 0, sizeof bp);
  const uint32_t need = c->D.Hkv >= 32 ? 0xFFFFFFFFu : ((1u << c->D.Hkv) - 1u);
  for (int s = 0; s < seq_count; ++s) {
    const size_t i = ls_index(c, layer, seq_begin + s);
    if (c->last_len[i] == 0) return fail(c, LTRI_ESTATE, "sequence %d: no chunk appended yet", seq_begin + s);
    if ((c->ever_sel[i] & need) != need)
      return fail(c, LTRI_ESTATE, "sequence %d: no earlier selection to keep (call ltri_retrieve once first)",
                  seq_begin + s);
    bp.seq[s] = seq_begin + s;
    bp.c0[s] = (int32_t)(c->n_tokens[i] - c->last_len[i]);
  }
  if (!c->dry) {
    r = check_hip(c, launch_persist_list(c->D, c->ds, layer, bp, seq_count, c->stream), "persistent selection");
    if (r != LTRI_OK) return r;
    r = fetch_retrieved(c, layer, bp, seq_count);
    if (r != LTRI_OK) return r;
  }
  for (int s = 0; s < seq_count; ++s) c->have_sel[ls_index(c, layer, seq_begin + s)] = 0xFFFFFFFFu;
  return LTRI_OK;
}

int32_t ltri_force_selection(ltri_ctx* c, int32_t layer, int32_t seq, int32_t kv_head, const int32_t* ids_host,
                             int32_t n) {
  int32_t r = check_range(c, layer, seq, 1);
  if (r != LTRI_OK) return r;
  if (kv_head < 0 || kv_head >= c->D.Hkv) return fail(c, LTRI_EINVAL, "kv_head %d out of range", kv_head);
  if (n < 0 || (n > 0 && !ids_host)) return fail(c, LTRI_EINVAL, "bad id list");
  const size_t i = ls_index(c, layer, seq);
  if (c->last_len[i] == 0) return fail(c, LTRI_ESTATE, "no chunk appended yet");
  std::vector<int32_t> ids(ids_host, ids_host + n);
  std::sort(ids.begin(), ids.end());
  ids.erase(std::unique(ids.begin(), ids.end()), ids.end());
  if (!ids.empty() && ids.front() < 0) return fail(c, LTRI_EINVAL, "negative span id");
  if ((long long)ids.size() > c->D.sel_cap)
    return fail(c, LTRI_ECAPACITY, "%zu ids exceed the selection capacity %d", ids.size(), c->D.sel_cap);
  if (!c->dry) {
    const int slot = (layer * c->D.n_seqs + seq) * c->D.Hkv + kv_head;
    if (!ids.empty()) {
      r = check_hip(c, hipMemcpyAsync(c->ds.sel_ids + (size_t)slot * c->D.sel_cap, ids.data(), ids.size() * 4,
                                      hipMemcpyHostToDevice, c->stream), "copy ids");
      if (r != LTRI_OK) return r;
      r = check_hip(c, hipStreamSynchronize(c->stream), "copy ids (sync)");
      if (r != LTRI_OK) return r;
    }
    r = check_hip(c, launch_force_list(c->D, c->ds, layer, seq, kv_head, (int)ids.size(), c->stream),
                  "forced selection");
    if (r != LTRI_OK) return r;
    BatchPos fb;
    memset(&fb, 0, sizeof fb);
    fb.seq[0] = seq;
    fb.c0[0] = (int32_t)(c->n_tokens[i] - c->last_len[i]);
    r = fetch_retrieved(c, layer, fb, 1);                 // every KV head of the sequence: the others' rows are fetched again
    if (r != LTRI_OK) return r;
  }
  c->have_sel[i] |= 1u << (kv_head & 31);
  c->ever_sel[i] |= 1u << (kv_head & 31);
  return LTRI_OK;
}

static int32_t attend_impl(ltri_ctx* c, int32_t layer, int32_t seq_begin, int32_t seq_count, const void* q, int32_t n_q,
                           void* out, float* lse, bool own_buffer) {
  BatchPos bp;
  memset(&bp, 0, sizeof bp);
  int32_t r = check_query_chunk(c, layer, seq_begin, seq_count, q, n_q, bp);
  if (r != LTRI_OK) return r;
  if (!out) return fail(c, LTRI_EINVAL, "out is NULL");
  const uint32_t need = c->D.Hkv >= 32 ? 0xFFFFFFFFu : ((1u << c->D.Hkv) - 1u);
  for (int s = 0; s < seq_count; ++s)
    if ((c->have_sel[ls_index(c, layer, seq_begin + s)] & need) != need)
      return fail(c, LTRI_ESTATE, "sequence %d: no selection for the last chunk (call ltri_retrieve first)",
                  seq_begin + s);
  float* part = c->dc.att_part;
  if (own_buffer) {
    // a dry context sizes the request for a device of 256 compute units
    const size_t bytes = attend_partial_bytes(c->D, seq_count, n_q, c->dry ? 256 : c->n_cus);
    if (bytes > ATT_STATIC_SCRATCH_BYTES)
      return fail(c, LTRI_ECAPACITY, "partial results of %d sequences x %d query rows take %zu bytes, the library's own buffer "
                  "holds %zu (use ltri_attend with the context's scratch)", seq_count, n_q, bytes, (size_t)ATT_STATIC_SCRATCH_BYTES);
    part = c->static_part;
  }
  if (!c->dry) {
    r = check_hip(c, launch_attend(c->D, c->ds, c->k_arena, c->v_arena, q, layer, bp, seq_count, n_q, out, lse,
                                   c->attend_stages, part, 0, nullptr, 0, nullptr, c->stream), "attend");
    if (r != LTRI_OK) return r;
  }
  return LTRI_OK;
}

int32_t ltri_attend(ltri_ctx* c, int32_t layer, int32_t seq_begin, int32_t seq_count, const void* q, int32_t n_q,
                    void* out, float* lse) {
  return attend_impl(c, layer, seq_begin, seq_count, q, n_q, out, lse, false);
}

int32_t ltri_attend_static(ltri_ctx* c, int32_t layer, int32_t seq_begin, int32_t seq_count, const void* q, int32_t n_q,
                           void* out, float* lse) {
  return attend_impl(c, layer, seq_begin, seq_count, q, n_q, out, lse, true);
}

// Next timing event of the context (created on first use), not recorded yet; NULL while timing is off.
static int32_t timing_event(ltri_ctx* c, hipEvent_t* ev) {
  *ev = nullptr;
  if (!c->step_timing) return LTRI_OK;
  if (c->tev_used == c->tev.size()) {
    hipEvent_t e = nullptr;
    // a device-scope release when recorded: nothing the host reads hangs on these events
    const int32_t r = check_hip(c, hipEventCreateWithFlags(&e, hipEventReleaseToDevice), "timing event");
    if (r != LTRI_OK) return r;
    c->tev.push_back(e);
  }
  *ev = c->tev[c->tev_used++];
  return LTRI_OK;
}
static int32_t timing_mark(ltri_ctx* c, hipStream_t s) {
  hipEvent_t e = nullptr;
  const int32_t r = timing_event(c, &e);
  if (r != LTRI_OK || !e) return r;
  return check_hip(c, hipEventRecord(e, s), "timing event");
}

// The timing events of one step: kept, with their count, when the step was queued whole; dropped otherwise.
struct StepTiming {
  ltri_ctx* c;
  size_t first;
  bool kept;
  explicit StepTiming(ltri_ctx* ctx) : c(ctx), first(ctx->tev_used), kept(false) {}
  void keep() {
    if (c->tev_used > first) c->tev_parts.push_back((uint8_t)(c->tev_used - first));
    kept = true;
  }
  ~StepTiming() { if (!kept) c->tev_used = first; }
};

int32_t ltri_set_step_timing(ltri_ctx* c, int32_t on) {
  if (!c) return LTRI_EINVAL;
  if (c->dry) return LTRI_OK;
  if (c->tev_used) {                      // drop the records of steps that were never read
    const int32_t r = check_hip(c, hipStreamSynchronize(c->stream), "synchronise");
    if (r != LTRI_OK) return r;
    c->tev_used = 0;
  }
  c->tev_parts.clear();
  c->step_timing = on != 0;
  return LTRI_OK;
}

int32_t ltri_read_step_timing(ltri_ctx* c, float* local_ms, float* retrieved_ms, int32_t cap, int32_t* n) {
  if (!c || !n || cap < 0 || (cap > 0 && (!local_ms || !retrieved_ms))) return LTRI_EINVAL;
  *n = 0;
  if (c->dry) return LTRI_OK;
  int32_t r = check_hip(c, hipStreamSynchronize(c->stream), "synchronise");
  if (r != LTRI_OK) return r;
  size_t e = 0;
  for (size_t i = 0; i < c->tev_parts.size() && (int32_t)i < cap; ++i) {
    r = check_hip(c, hipEventElapsedTime(&local_ms[i], c->tev[e], c->tev[e + 1]), "timing");
    retrieved_ms[i] = 0.0f;
    if (r == LTRI_OK && c->tev_parts[i] == 4)
      r = check_hip(c, hipEventElapsedTime(&retrieved_ms[i], c->tev[e + 2], c->tev[e + 3]), "timing");
    if (r != LTRI_OK) return r;
    e += c->tev_parts[i];
    ++*n;
  }
  c->tev_used = 0;
  c->tev_parts.clear();
  return LTRI_OK;
}

int32_t ltri_step(ltri_ctx* c, int32_t layer, int32_t seq_begin, int32_t seq_count, const void* k_chunk,
                  const void* v_chunk, const void* q_seg, const void* q, int32_t n_new, void* out, float* lse) {
  if (!c) return LTRI_EINVAL;
  if (!q) return fail(c, LTRI_EINVAL, "q is NULL");
  if (!out) return fail(c, LTRI_EINVAL, "out is NULL");
  // Short query blocks (decode) and shapes the matrix-core kernel does not take go through the three calls.
  const bool overlap = !c->dry && n_new > ATT_SPLIT_MAX_ROWS && attend_on_matrix_cores(c->D) && seq_count >= 1 &&
                       seq_count <= LTRI_MAX_BATCH;
  if (!overlap && !c->dry && n_new == 1) {
    // Decode: steps 1 and 2 of a one-token chunk in one launch where that kernel applies, then step 3.
    BatchPos bp;
    memset(&bp, 0, sizeof bp);
    int32_t r = append_common(c, layer, seq_begin, seq_count, k_chunk, v_chunk, 1, bp);
    if (r != LTRI_OK) return r;
    long long bound = 0;
    for (int s = 0; s < seq_count; ++s)
      bound = std::max(bound, std::min<long long>(c->span_bound[ls_index(c, layer, seq_begin + s)] + 1, c->D.max_spans));
    if (retrieve_is_one_launch(c->D, 1, (int)bound)) {
      append_commit(c, layer, seq_begin, seq_count, 1);
      r = check_hip(c, launch_retrieve(c->D, c->ds, c->dc, c->CL.max_problems, q, layer, bp, seq_count, 1, (int)bound,
                                       nullptr, nullptr, nullptr, c->k_arena, nullptr, false, c->stream), "append and retrieve (one token)");
      if (r != LTRI_OK) return r;
      r = fetch_retrieved(c, layer, bp, seq_count);
      if (r != LTRI_OK) return r;
      for (int s = 0; s < seq_count; ++s) {
        c->have_sel[ls_index(c, layer, seq_begin + s)] = 0xFFFFFFFFu;
        c->ever_sel[ls_index(c, layer, seq_begin + s)] = 0xFFFFFFFFu;
      }
    } else {
      r = append_spans(c, layer, bp, seq_count, q_seg, 1, nullptr);
      if (r != LTRI_OK) return r;
      append_commit(c, layer, seq_begin, seq_count, 1);
      r = ltri_retrieve(c, layer, seq_begin, seq_count, q, 1, nullptr, nullptr);
      if (r != LTRI_OK) return r;
    }
    return ltri_attend(c, layer, seq_begin, seq_count, q, 1, out, lse);
  }
  if (!overlap) {
    int32_t r = ltri_append_chunk(c, layer, seq_begin, seq_count, k_chunk, v_chunk, q_seg, n_new);
    if (r != LTRI_OK) return r;
    r = ltri_retrieve(c, layer, seq_begin, seq_count, q, n_new, nullptr, nullptr);
    if (r != LTRI_OK) return r;
    return ltri_attend(c, layer, seq_begin, seq_count, q, n_new, out, lse);
  }
  BatchPos bp;
  memset(&bp, 0, sizeof bp);
  int32_t r = append_common(c, layer, seq_begin, seq_count, k_chunk, v_chunk, n_new, bp);
  if (r != LTRI_OK) return r;
  const bool keys_with_step2 = retrieve_stores_rep_keys(c->D, n_new);
  StepTiming timing(c);
  bool sums_ready = false;               // step 2's running sums of the query and key rows ride in step 1's first launch
  if (!c->D.offload) {
    // Keys and values resident on the device: the three steps follow each other on the context's stream and the
    // attention is one launch over initial | retrieved | window | chunk. Its workgroups are equal in work (row
    // sub-tiles paired from both ends of the chunk) and fill every compute unit, so a split that runs the first
    // part beside the small kernels of steps 1 and 2 only makes those wait for a free compute unit.
    r = append_spans(c, layer, bp, seq_count, q_seg, n_new, nullptr, keys_with_step2, q, &sums_ready);
    if (r != LTRI_OK) return r;
    append_commit(c, layer, seq_begin, seq_count, n_new);
    r = retrieve_impl(c, layer, seq_begin, seq_count, q, n_new, nullptr, nullptr, keys_with_step2, sums_ready);
    if (r != LTRI_OK) return r;
    hipEvent_t t_begin = nullptr, t_end = nullptr;     // the attention launch carries its timing events itself
    r = timing_event(c, &t_begin);
    if (r == LTRI_OK) r = timing_event(c, &t_end);
    if (r != LTRI_OK) return r;
    r = check_hip(c, launch_attend(c->D, c->ds, c->k_arena, c->v_arena, q, layer, bp, seq_count, n_new, out, lse,
                                   c->attend_stages, c->dc.att_part, 0, nullptr, 0, nullptr, c->stream, t_begin, t_end),
                  "attend");
    if (r == LTRI_OK) timing.keep();
    return r;
  }
  // Keys and values in host memory: the rows of the retrieved tokens cross the host link after step 2, which takes
  // longer than anything else in the step. That fetch runs on a second stream; the attention over initial | window
  // | chunk follows step 2 on the context's stream, beside the fetch, and the launch over the retrieved rows, behind
  // the join, folds its result in. (The attention stays on the stream whose kernels precede it: once the fetch
  // fills the host link, a launch on another stream starts 100-200 us late. Measured alternatives: beside the small
  // kernels of steps 1 and 2 the first part holds every compute unit's LDS and step 2's last launch waits for it to
  // end; and the chunk's rows written out to the host beside step 1, by a kernel of any size or by copies, slow
  // step 1's kernels by as much as the overlap gains: 21 -> 140 us for the first tile kernel.)
  float* lse_a = c->dc.att_lse2;
  bool side_queued = false;
  auto both_streams = [&]() -> int32_t {
    int32_t e = check_hip(c, launch_local_list(c->D, bp, seq_count, c->dc.loclist, c->CL.loc_cap, c->stream), "local list");
    if (e != LTRI_OK) return e;
    e = append_spans(c, layer, bp, seq_count, q_seg, n_new, nullptr, keys_with_step2, q, &sums_ready);
    if (e != LTRI_OK) return e;
    append_commit(c, layer, seq_begin, seq_count, n_new);
    side_queued = true;                  // (from here on the second stream may hold work of this step)
    e = retrieve_impl(c, layer, seq_begin, seq_count, q, n_new, nullptr, nullptr, keys_with_step2, sums_ready, c->ev_fork,
                      c->side);
    if (e != LTRI_OK) return e;
    e = timing_mark(c, c->stream);
    if (e == LTRI_OK)
      e = check_hip(c, launch_attend(c->D, c->ds, c->k_arena, c->v_arena, q, layer, bp, seq_count, n_new, out, lse_a,
                                     c->step_stages, nullptr, 1, c->dc.loclist, c->CL.loc_cap, nullptr, c->stream),
                    "attend (initial, window, chunk)");
    if (e == LTRI_OK) e = timing_mark(c, c->stream);
    return e;
  };
  r = both_streams();
  // The join, then the retrieved tokens, whose launch folds the first part's result into its own. Join even after an
  // error, so that the context's stream never runs ahead of the second stream's writes.
  int32_t rj = LTRI_OK;
  if (side_queued) {
    rj = check_hip(c, hipEventRecord(c->ev_join, c->side), "join");
    if (rj == LTRI_OK) rj = check_hip(c, hipStreamWaitEvent(c->stream, c->ev_join, 0), "join");
  }
  if (r != LTRI_OK) return r;
  if (rj != LTRI_OK) return rj;
  r = timing_mark(c, c->stream);
  if (r != LTRI_OK) return r;
  r = check_hip(c, launch_attend(c->D, c->ds, c->k_arena, c->v_arena, q, layer, bp, seq_count, n_new, out, lse,
                                 c->step_stages, nullptr, 2, nullptr, 0, lse_a, c->stream),
                "attend (retrieved)");
  if (r != LTRI_OK) return r;
  r = timing_mark(c, c->stream);
  if (r == LTRI_OK) timing.keep();
  return r;
}

int32_t ltri_gather_pack(ltri_ctx* c, int32_t layer, int32_t seq, void* k_packed, void* v_packed,
                         int32_t* n_tokens) {
  int32_t r = check_range(c, layer, seq, 1);
  if (r != LTRI_OK) return r;
  if (!k_packed || !v_packed) return fail(c, LTRI_EINVAL, "packed buffers missing");
  const size_t i = ls_index(c, layer, seq);
  const uint32_t need = c->D.Hkv >= 32 ? 0xFFFFFFFFu : ((1u << c->D.Hkv) - 1u);
  if (c->last_len[i] == 0 || (c->have_sel[i] & need) != need) return fail(c, LTRI_ESTATE, "no selection to gather");
  if (!c->dry) {
    r = check_hip(c, launch_gather_pack(c->D, c->ds, c->k_arena, c->v_arena, layer, seq, k_packed, v_packed,
                                        n_tokens, c->stream), "gather");
    if (r != LTRI_OK) return r;
  }
  return LTRI_OK;
}

// ---- introspection ----
static int32_t check_slot(ltri_ctx* c, int layer, int seq, int h) {
  int32_t r = check_range(c, layer, seq, 1);
  if (r != LTRI_OK) return r;
  if (h < 0 || h >= c->D.Hkv) return fail(c, LTRI_EINVAL, "kv_head %d out of range", h);
  if (c->dry) return fail(c, LTRI_ESTATE, "no device data in dry-run mode");
  return check_hip(c, hipStreamSynchronize(c->stream), "synchronise");
}

static int32_t read_dev(ltri_ctx* c, void* dst, const void* src, size_t bytes) {
  if (bytes == 0) return LTRI_OK;
  return check_hip(c, hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost), "read back");
}

int32_t ltri_sync_status(ltri_ctx* c) {
  if (!c) return LTRI_EINVAL;
  if (c->dry) return LTRI_OK;
  int32_t r = check_hip(c, hipStreamSynchronize(c->stream), "synchronise");
  if (r != LTRI_OK) return r;
  int32_t e[4] = {0, 0, 0, 0};
  r = read_dev(c, e, c->ds.err, sizeof e);
  if (r != LTRI_OK) return r;
  if (e[0] != 0) return fail(c, e[0], "raised on the device: %s", ltri_strerror(e[0]));
  return LTRI_OK;
}

int32_t ltri_token_count(ltri_ctx* c, int32_t layer, int32_t seq, int64_t* n) {
  int32_t r = check_range(c, layer, seq, 1);
  if (r != LTRI_OK) return r;
  if (!n) return LTRI_EINVAL;
  *n = c->n_tokens[ls_index(c, layer, seq)];
  return LTRI_OK;
}

static int32_t read_meta(ltri_ctx* c, int layer, int seq, int h, int32_t* meta) {
  const int slot = (layer * c->D.n_seqs + seq) * c->D.Hkv + h;
  return read_dev(c, meta, c->ds.meta + (size_t)slot * META_WORDS, META_WORDS * 4);
}

int32_t ltri_span_count(ltri_ctx* c, int32_t layer, int32_t seq, int32_t h, int32_t* n) {
  int32_t r = check_slot(c, layer, seq, h);
  if (r != LTRI_OK) return r;
  if (!n) return LTRI_EINVAL;
  int32_t meta[META_WORDS];
  r = read_meta(c, layer, seq, h, meta);
  if (r != LTRI_OK) return r;
  *n = meta[META_N_SPANS];
  return LTRI_OK;
}

int32_t ltri_get_spans(ltri_ctx* c, int32_t layer, int32_t seq, int32_t h, int32_t* starts_host,
                       int32_t* lens_host, int32_t cap) {
  int32_t r = check_slot(c, layer, seq, h);
  if (r != LTRI_OK) return r;
  int32_t meta[META_WORDS];
  r = read_meta(c, layer, seq, h, meta);
  if (r != LTRI_OK) return r;
  const int n = std::min(meta[META_N_SPANS], cap);
  if (n < 0) return LTRI_EINVAL;
  const int slot = (layer * c->D.n_seqs + seq) * c->D.Hkv + h;
  if (starts_host) { r = read_dev(c, starts_host, c->ds.span_start + (size_t)slot * c->D.max_spans, (size_t)n * 4); if (r) return r; }
  if (lens_host) { r = read_dev(c, lens_host, c->ds.span_len + (size_t)slot * c->D.max_spans, (size_t)n * 4); if (r) return r; }
  return LTRI_OK;
}

int32_t ltri_get_rep_keys(ltri_ctx* c, int32_t layer, int32_t seq, int32_t h, void* reps_host, int32_t cap) {
  int32_t r = check_slot(c, layer, seq, h);
  if (r != LTRI_OK) return r;
  if (!reps_host) return LTRI_EINVAL;
  int32_t meta[META_WORDS];
  r = read_meta(c, layer, seq, h, meta);
  if (r != LTRI_OK) return r;
  const int n = std::min(meta[META_N_SPANS], cap);
  if (n < 0) return LTRI_EINVAL;
  const int slot = (layer * c->D.n_seqs + seq) * c->D.Hkv + h;
  const size_t row = (size_t)c->D.d * c->D.elt;
  return read_dev(c, reps_host, (char*)c->ds.krep + (size_t)slot * c->D.max_spans * row, (size_t)n * row);
}

int32_t ltri_get_selection(ltri_ctx* c, int32_t layer, int32_t seq, int32_t h, int32_t* ids_host, int32_t cap,
                           int32_t* n, double* scores_host) {
  int32_t r = check_slot(c, layer, seq, h);
  if (r != LTRI_OK) return r;
  int32_t meta[META_WORDS];
  r = read_meta(c, layer, seq, h, meta);
  if (r != LTRI_OK) return r;
  const int slot = (layer * c->D.n_seqs + seq) * c->D.Hkv + h;
  const int cnt = meta[META_SEL_CNT];
  if (n) *n = cnt;
  if (ids_host) { r = read_dev(c, ids_host, c->ds.sel_ids + (size_t)slot * c->D.sel_cap, (size_t)std::max(0, std::min(cnt, cap)) * 4); if (r) return r; }
  if (scores_host) { r = read_dev(c, scores_host, c->ds.scores + (size_t)slot * c->D.max_spans, (size_t)meta[META_N_SPANS] * 8); if (r) return r; }
  return LTRI_OK;
}

int32_t ltri_get_token_list(ltri_ctx* c, int32_t layer, int32_t seq, int32_t h, int32_t* tokens_host, int32_t cap,
                            int32_t* n) {
  int32_t r = check_slot(c, layer, seq, h);
  if (r != LTRI_OK) return r;
  int32_t meta[META_WORDS];
  r = read_meta(c, layer, seq, h, meta);
  if (r != LTRI_OK) return r;
  const int slot = (layer * c->D.n_seqs + seq) * c->D.Hkv + h;
  const int len = meta[META_LIST_LEN];
  if (n) *n = len;
  if (tokens_host) return read_dev(c, tokens_host, c->ds.tok_list + (size_t)slot * c->D.list_cap, (size_t)std::max(0, std::min(len, cap)) * 4);
  return LTRI_OK;
}

int32_t ltri_get_index_tokens(ltri_ctx* c, int32_t layer, int32_t seq, int32_t h, uint32_t* mask_host,
                              int32_t cap_words) {
  int32_t r = check_slot(c, layer, seq, h);
  if (r != LTRI_OK) return r;
  if (c->D.rep_mode != LTRI_REP_DYNAMIC) return fail(c, LTRI_ESTATE, "the context stores mean representatives");
  const int len = c->last_len[ls_index(c, layer, seq)];
  if (len == 0) return fail(c, LTRI_ESTATE, "no chunk appended yet");
  const int words = (len + 31) / 32;
  if (!mask_host || cap_words < words) return fail(c, LTRI_EINVAL, "mask_host holds %d words, %d needed", cap_words, words);
  if (len == 1) { mask_host[0] = 1u; return LTRI_OK; }     // a one-token chunk is its own index token
  const int slot = (layer * c->D.n_seqs + seq) * c->D.Hkv + h;
  return read_dev(c, mask_host, c->ds.idx_mask + (size_t)slot * IDX_MASK_WORDS, (size_t)words * 4);
}

int32_t ltri_get_theta(ltri_ctx* c, int32_t layer, int32_t seq, int32_t h, double* theta_host) {
  int32_t r = check_slot(c, layer, seq, h);
  if (r != LTRI_OK) return r;
  if (!theta_host) return fail(c, LTRI_EINVAL, "theta_host is NULL");
  if (c->dry) return fail(c, LTRI_ESTATE, "a dry context runs no kernels");
  if (!(c->D.theta_quantile > 0.0)) return fail(c, LTRI_ESTATE, "the context uses an absolute threshold");
  if (c->last_len[ls_index(c, layer, seq)] <= 1) return fail(c, LTRI_ESTATE, "no chunk of more than one token appended last");
  if (layer != c->theta_layer || seq < c->theta_seq0 || seq >= c->theta_seq0 + c->theta_seqs)
    return fail(c, LTRI_ESTATE, "the device holds the thresholds of layer %d, sequences %d .. %d only", c->theta_layer,
                c->theta_seq0, c->theta_seq0 + c->theta_seqs - 1);
  const size_t p = (size_t)(seq - c->theta_seq0) * c->D.Hkv + h;
  return read_dev(c, theta_host, c->dc.qstate + p * QUANT_STATE_WORDS + 2, sizeof(double));
}

}  // extern "C"
