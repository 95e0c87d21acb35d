// Step 2 on the device (Sec. 3.4 second step): query-span representatives, similarity of
// every stored span with them (Eq. 8 with one vector per span, max over the query spans as in
// Eq. 9), budgeted top-k selection, and the flat list of context tokens
// (initial | retrieved | window) that step 3 reads.
//
// Scores are accumulated in fp64: products of bf16 (or fp32) values are exact in fp64, so the
// order of the selection does not depend on the summation order of any implementation.
#include <cstring>
#include <type_traits>
#include "device_common.h"
#include "span_mean.h"
#include "running_sums.h"

namespace ltri {

struct RetArgs {
  Dims D; DevState st; DevScratch sc; const void* q;
  int layer; int seq_count; int n_q; int Lp;
  int batch_off; int units_cap;          // two-stage query representatives (long chunks)
  int32_t* sel_ids_out; int32_t* sel_cnt_out;
  const void* k_arena; int append_first;  // one-token chunk: step 1 (the token becomes a span of its own) in the same launch
  const void* rep_k_arena;                // not NULL: the launch of the query-span pieces also stores the chunk's mean keys
  int qrep_by_last;                       // the last workgroup of the pieces' launch adds them up into Q^R
  int ticket_base;                        // first ticket counter of retrieve_chunk_kernel's problems
  int qrep_from_sums;                     // retrieve_chunk_kernel builds Q^R (and, with rs.k_arena, the chunk's mean keys)
  RunSums rs;                             // itself from these running sums
  BatchPos bp;
};

// Dynamic index vectors: the mask of the chunk's index tokens (bit = chunk-local token), or
// nullptr when every token counts (mean representatives; a one-token chunk is its own index token).
__device__ __forceinline__ const uint32_t* index_mask(const Dims& D, const DevState& st, int slot, const int32_t* meta) {
  if (D.rep_mode != LTRI_REP_DYNAMIC || meta[META_CHUNK_LEN] <= 1) return nullptr;
  return st.idx_mask + (size_t)slot * IDX_MASK_WORDS;
}

// ---- Q^R: mean over each query span of the group-summed query rows (dynamic index vectors:
//      their sum over the span's index tokens) ----
template <int DT>
__global__ __launch_bounds__(1024) void qrep_kernel(RetArgs a) {
  typedef typename Elt<DT>::type T;
  __shared__ double part[16][128];
  const Dims& D = a.D;
  const int p = blockIdx.y, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int first = meta[META_CHUNK_FIRST], nsp = meta[META_CHUNK_NSP], c0 = meta[META_CHUNK_START];
  const int d = D.d;
  const T* Qb = reinterpret_cast<const T*>(a.q) + (size_t)bi * a.n_q * D.Hq * d + (size_t)h * D.G * d;
  T* out = reinterpret_cast<T*>(a.sc.qrep) + (size_t)p * a.Lp * d;
  for (int qs = blockIdx.x; qs < nsp; qs += gridDim.x) {
    const int sid = first + qs;
    const int start = a.st.span_start[(size_t)slot * D.max_spans + sid] - c0;   // chunk-local
    const int len = a.st.span_len[(size_t)slot * D.max_spans + sid];
    span_mean_block<DT>(Qb + (size_t)start * D.Hq * d, (size_t)D.Hq * d, D.G, len, d, out + (size_t)qs * d, part,
                        nullptr, index_mask(D, a.st, slot, meta), start);
  }
}

// Long chunks: a query span is cut into pieces of QREP_PIECE tokens, one workgroup per piece
// (so that a 1024-token span is read by eight compute units instead of one); a second kernel
// adds the pieces of every span in ascending order.
constexpr int QREP_PIECE = 128;

// Piece u of the chunk's spans -> (span q, first token, token count); returns false past the end.
// Called by whole wavefronts with the same u: the spans' piece counts are scanned 64 at a time
// across the lanes (one load per lane instead of a serial walk over the table).
__device__ __forceinline__ bool qrep_unit(const int32_t* slen, int nsp, int u, int& q, int& t0, int& nt) {
  const int lane = threadIdx.x & 63;
  int base = 0;
  for (int q0 = 0; q0 < nsp; q0 += 64) {
    const int ql = q0 + lane;
    const int len = ql < nsp ? slen[ql] : 0;
    const int parts = (len + QREP_PIECE - 1) / QREP_PIECE;
    int incl = parts;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o, 64);
      if (lane >= o) incl += v;
    }
    const int total = __shfl(incl, 63, 64);
    if (u < base + total) {
      const int src = __ffsll((long long)__ballot(u < base + incl)) - 1;    // first span whose pieces reach past u
      q = q0 + src;
      t0 = (u - base - __shfl(incl - parts, src, 64)) * QREP_PIECE;
      nt = min(QREP_PIECE, __shfl(len, src, 64) - t0);
      return true;
    }
    base += total;
  }
  return false;
}

// Pieces before span q (same scan).
__device__ __forceinline__ int qrep_first_unit(const int32_t* slen, int q) {
  const int lane = threadIdx.x & 63;
  int base = 0;
  for (int q0 = 0; q0 < q; q0 += 64) {
    const int ql = q0 + lane;
    const int parts = ql < q ? (slen[ql] + QREP_PIECE - 1) / QREP_PIECE : 0;
    int sum = parts;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    base += sum;
  }
  return base;
}

constexpr int QREP_GRID_X = 64;            // workgroups per problem that walk the pieces

template <int DT>
__global__ __launch_bounds__(1024) void qrep_partial_kernel(RetArgs a) {
  typedef typename Elt<DT>::type T;
  __shared__ double part[16][128];
  const Dims& D = a.D;
  const int p = blockIdx.y, bi = a.batch_off + p / D.Hkv, h = p % D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int first = meta[META_CHUNK_FIRST], nsp = meta[META_CHUNK_NSP], c0 = meta[META_CHUNK_START];
  const int d = D.d;
  if (blockIdx.x >= QREP_GRID_X) {
    // The workgroups beyond the pieces' own: the mean keys of the chunk's spans (Sec. 3.3.1), which nothing in
    // this step reads (the chunk's spans lie inside the window), so they ride along instead of taking a launch.
    if (!a.rep_k_arena) return;
    const T* Kb = reinterpret_cast<const T*>(a.rep_k_arena) + arena_off(D, slot);
    for (int q = blockIdx.x - QREP_GRID_X; q < nsp; q += gridDim.x - QREP_GRID_X) {
      const int sid = first + q;
      const int start = a.st.span_start[(size_t)slot * D.max_spans + sid];
      const int len = a.st.span_len[(size_t)slot * D.max_spans + sid];
      T* rep = reinterpret_cast<T*>(a.st.krep) + ((size_t)slot * D.max_spans + sid) * d;
      span_mean_block<DT>(Kb + (size_t)chunk_tok_row(D, c0, start) * d, (size_t)d, 1, len, d, rep, part);
    }
    return;
  }
  const T* Qb = reinterpret_cast<const T*>(a.q) + (size_t)bi * a.n_q * D.Hq * d + (size_t)h * D.G * d;
  const int32_t* slen = a.st.span_len + (size_t)slot * D.max_spans + first;
  const int32_t* sstart = a.st.span_start + (size_t)slot * D.max_spans + first;
  double* psum = a.sc.qpart + (size_t)p * a.units_cap * d;
  for (int u = blockIdx.x; u < a.units_cap; u += QREP_GRID_X) {
    int q, t0, nt;
    if (!qrep_unit(slen, nsp, u, q, t0, nt)) break;            // uniform over the block
    const int start = sstart[q] - c0 + t0;                      // chunk-local
    span_mean_block<DT>(Qb + (size_t)start * D.Hq * d, (size_t)D.Hq * d, D.G, nt, d, nullptr, part,
                        psum + (size_t)u * d, index_mask(D, a.st, slot, meta), start);
  }
  if (!a.qrep_by_last) return;
  // The workgroup of a problem that finishes last adds the pieces up into Q^R and leaves the ticket counter at
  // zero for the next launch. The sums are stored and loaded at device scope (they bypass the caches that the
  // compute units of one die do not share with the others), every store of a workgroup has completed at the
  // barrier before its ticket is taken, and the ticket is a device-scope atomic: no device-wide fence, which
  // would write back and invalidate the whole level-2 cache, is needed.
  __shared__ int s_last;
  __syncthreads();
  if (threadIdx.x == 0) s_last = atomicAdd(&a.sc.tickets[p], 1) == QREP_GRID_X - 1;
  __syncthreads();
  if (!s_last) return;
  T* qrep = reinterpret_cast<T*>(a.sc.qrep) + (size_t)(bi * D.Hkv + h) * a.Lp * d;
  const bool summed = index_mask(D, a.st, slot, meta) != nullptr;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int q = wave; q < nsp; q += 16) {                  // the pieces of a span in ascending order, one wavefront per span
    const int u0 = qrep_first_unit(slen, q);
    const int len = slen[q];
    const int parts = (len + QREP_PIECE - 1) / QREP_PIECE;
    for (int c = lane; c < d; c += 64) {
      double sum = 0.0;
      for (int k = 0; k < parts; ++k)
        sum += __hip_atomic_load(psum + (size_t)(u0 + k) * d + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      qrep[(size_t)q * d + c] = Elt<DT>::from_f64(summed ? sum : sum / (double)len);
    }
  }
  if (threadIdx.x == 0) a.sc.tickets[p] = 0;
}

// ---- long chunks, mean representatives: the running sums as a launch of their own (when the segmentation's
//      first launch has not taken them along) ----
template <int DT>
__global__ __launch_bounds__(1024) void running_sums_kernel(RetArgs a) {
  __shared__ double wt[16 * 16 * 8];
  running_sums_block<DT, 16>(a.D, a.bp, a.layer, a.batch_off, a.rs, blockIdx.x, blockIdx.y, wt);
}

template <int DT>
__global__ __launch_bounds__(128) void qrep_final_kernel(RetArgs a) {
  typedef typename Elt<DT>::type T;
  const Dims& D = a.D;
  const int p = blockIdx.y, bi = a.batch_off + p / D.Hkv, h = p % D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int first = meta[META_CHUNK_FIRST], nsp = meta[META_CHUNK_NSP];
  const int d = D.d, c = threadIdx.x;
  const int32_t* slen = a.st.span_len + (size_t)slot * D.max_spans + first;
  const double* psum = a.sc.qpart + (size_t)p * a.units_cap * d;
  T* out = reinterpret_cast<T*>(a.sc.qrep) + (size_t)(bi * D.Hkv + h) * a.Lp * d;
  if (c >= d) return;
  for (int q = blockIdx.x; q < nsp; q += gridDim.x) {
    const int u0 = qrep_first_unit(slen, q);
    const int len = slen[q];
    const int parts = (len + QREP_PIECE - 1) / QREP_PIECE;
    double s = 0.0;
    for (int k = 0; k < parts; ++k) s += psum[(size_t)(u0 + k) * d + c];
    out[(size_t)q * d + c] = Elt<DT>::from_f64(index_mask(D, a.st, slot, meta) ? s : s / (double)len);
  }
}

// ---- score_i = max_j Qrep_j . Krep_i for every stored span ----
// Four lanes per stored span, each over a quarter of the 16-byte pieces of its representative key;
// the query representatives are staged in LDS as doubles, sixteen at a time. Products of the stored values are exact in
// fp64 and 128 of them are summed, so the order of the sum does not matter at the 1e-12 level
// the selection is compared at.
constexpr int SCORE_QBATCH = 16;
template <int DT>
__global__ __launch_bounds__(256) void score_kernel(RetArgs a) {
  typedef typename Elt<DT>::type T;
  constexpr int N = 16 / (int)sizeof(T);                // elements per 16-byte piece
  extern __shared__ double qs[];                      // [SCORE_QBATCH][d]
  const Dims& D = a.D;
  const int p = blockIdx.y, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int n = meta[META_N_SPANS], nqs = meta[META_CHUNK_NSP];
  if ((int)(blockIdx.x * (blockDim.x / 4)) >= n) return;    // uniform
  const int d = D.d;
  const T* qrep = reinterpret_cast<const T*>(a.sc.qrep) + (size_t)p * a.Lp * d;
  const T* krep = reinterpret_cast<const T*>(a.st.krep) + (size_t)slot * D.max_spans * d;
  double* scores = a.st.scores + (size_t)slot * D.max_spans;
  const int i = blockIdx.x * (blockDim.x / 4) + (threadIdx.x >> 2), part = threadIdx.x & 3;
  const uint4* krow = reinterpret_cast<const uint4*>(krep + (size_t)max(min(i, n - 1), 0) * d);
  // the lane's pieces of the key are requested before the query representatives are staged
  constexpr int MAXP = 128 / N / 4;                     // pieces per lane at d = 128
  uint4 kv[MAXP];
#pragma unroll
  for (int q = 0; q < MAXP; ++q) kv[q] = (part + 4 * q < d / N) ? krow[part + 4 * q] : make_uint4(0u, 0u, 0u, 0u);
  double best = -INFINITY;
  for (int j0 = 0; j0 < nqs; j0 += SCORE_QBATCH) {
    const int nj = min(SCORE_QBATCH, nqs - j0);
    __syncthreads();
    for (int q = threadIdx.x; q < nj * d; q += blockDim.x) qs[q] = Elt<DT>::to_f64(qrep[(size_t)j0 * d + q]);
    __syncthreads();
    double acc[SCORE_QBATCH];
#pragma unroll
    for (int jj = 0; jj < SCORE_QBATCH; ++jj) acc[jj] = 0.0;
#pragma unroll
    for (int q = 0; q < MAXP; ++q) {
      const int pc = part + 4 * q;
      if (pc < d / N) {
        double k[8];
        if constexpr (DT == LTRI_BF16) {
          const uint32_t w[4] = {kv[q].x, kv[q].y, kv[q].z, kv[q].w};
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            k[2 * u] = (double)__uint_as_float(w[u] << 16);
            k[2 * u + 1] = (double)__uint_as_float(w[u] & 0xffff0000u);
          }
        } else {
          k[0] = (double)__uint_as_float(kv[q].x); k[1] = (double)__uint_as_float(kv[q].y);
          k[2] = (double)__uint_as_float(kv[q].z); k[3] = (double)__uint_as_float(kv[q].w);
        }
#pragma unroll
        for (int jj = 0; jj < SCORE_QBATCH; ++jj) {
          if (jj < nj) {
#pragma unroll
            for (int u = 0; u < N; ++u) acc[jj] = fma(k[u], qs[jj * d + pc * N + u], acc[jj]);
          }
        }
      }
    }
#pragma unroll
    for (int jj = 0; jj < SCORE_QBATCH; ++jj) {
      double v = acc[jj];
      v += __shfl_xor(v, 1, 64);
      v += __shfl_xor(v, 2, 64);
      if (jj < nj) best = fmax(best, v);
    }
  }
  if (i < n && part == 0) scores[i] = best;
}

// ---- scores on the matrix cores, in fp64 ----
// best[v] = max_j Q^R_j . K^R_i for the four spans i = i0 + 4 v + lane / 16 of a tile of 16 spans, by one
// wavefront: D (16 spans x 16 query spans) = A (16 x d) B (d x 16) as d / 4 products v_mfma_f64_16x16x4f64.
// The stored values are converted to fp64 exactly and their products are exact in fp64, so the scores differ
// from any other fp64 evaluation only by the order of the 128 additions (Eq. 8; the selection is compared at
// 1e-12). A lane (r = lane % 16, g = lane / 16) feeds row r of A (span i0 + r) and column r of B (query span
// j0 + r): both fetch the 16-byte pieces g, g + 4, ... of their row, and product step (t, e) takes element e of
// piece g + 4 t from either side, i.e. the same k on both sides in a permuted order. Rows past n and columns
// past nqs read a valid row and are masked. All 64 lanes must call it together.
typedef double f64x4_t __attribute__((ext_vector_type(4)));
template <int DT>
__device__ __forceinline__ void score_tile_f64(const typename Elt<DT>::type* krep, int n, int i0,
                                               const typename Elt<DT>::type* qrep, int nqs, int d, double (&best)[4]) {
  typedef typename Elt<DT>::type T;
  constexpr int N = 16 / (int)sizeof(T);                // elements per 16-byte piece
  constexpr int TMAX = 128 * (int)sizeof(T) / 16 / 4;   // pieces per lane at d = 128
  const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int nt = d / N / 4;                             // pieces per lane
  const uint4* arow = reinterpret_cast<const uint4*>(krep + (size_t)max(min(i0 + r, n - 1), 0) * d);
  uint4 av[TMAX];
#pragma unroll
  for (int t = 0; t < TMAX; ++t) av[t] = t < nt ? arow[g + 4 * t] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
  for (int v = 0; v < 4; ++v) best[v] = -INFINITY;
  auto elem = [](const uint4& u, int e) -> double {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
    if constexpr (DT == LTRI_BF16) return (double)__uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16));
    else return (double)__uint_as_float(w[e]);
  };
  for (int j0 = 0; j0 < nqs; j0 += 16) {
    const uint4* brow = reinterpret_cast<const uint4*>(qrep + (size_t)min(j0 + r, nqs - 1) * d);
    uint4 bv[TMAX];
#pragma unroll
    for (int t = 0; t < TMAX; ++t) bv[t] = t < nt ? brow[g + 4 * t] : make_uint4(0u, 0u, 0u, 0u);
    f64x4_t acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int t = 0; t < TMAX; ++t) {
      if (t < nt) {
#pragma unroll
        for (int e = 0; e < N; ++e) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(elem(av[t], e), elem(bv[t], e), acc, 0, 0, 0);
      }
    }
    // acc[v] = score of span i0 + 4 v + g against query span j0 + r: maximum over the 16 lanes of a group
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      double m = (j0 + r < nqs) ? acc[v] : -INFINITY;
      m = fmax(m, __shfl_xor(m, 1, 64));
      m = fmax(m, __shfl_xor(m, 2, 64));
      m = fmax(m, __shfl_xor(m, 4, 64));
      m = fmax(m, __shfl_xor(m, 8, 64));
      best[v] = fmax(best[v], m);
    }
  }
}

// Evicted part [a, b) of a stored span for a chunk starting at c0.
__device__ __forceinline__ void clip_span(const Dims& D, int c0, int start, int len, int& a, int& b) {
  const int ns = min(D.n_sink, c0);
  const int ws = max(ns, c0 - D.window);
  a = max(start, ns);
  b = min(start + len, ws);
}

// Items a selection ranges over: the stored spans, or (retrieval by memory units) the units that
// hold the tokens stored so far.
__device__ __forceinline__ int item_count(const Dims& D, const int32_t* meta) {
  if (D.unit > 0) return (meta[META_CHUNK_START] + meta[META_CHUNK_LEN] + D.unit - 1) / D.unit;
  return meta[META_N_SPANS];
}

// Token range of item i of the selection: a stored span, or (retrieval by memory units) unit i.
__device__ __forceinline__ void item_range(const Dims& D, const int32_t* sstart, const int32_t* slen,
                                           int n_tokens, int i, int& start, int& len) {
  if (D.unit > 0) {
    start = i * D.unit;
    len = min(D.unit, n_tokens - start);
  } else {
    start = sstart[i];
    len = slen[i];
  }
}

// Given the selection as a bit mask over item ids (spans, or units), writes the ascending id list,
// the token list and their lengths. Called by all 1024 threads of the block.
constexpr int EMIT_CAP = 2048;     // selected spans whose tokens are written cooperatively

__device__ __forceinline__ void emit_selection(const Dims& D, const DevState& st, int slot, const uint32_t* selmask,
                               int n, int32_t* ids_out, int32_t* cnt_out) {
  __shared__ int s_wcnt[16], s_wtok[16], s_base_cnt, s_base_tok;
  __shared__ int e_a[EMIT_CAP], e_len[EMIT_CAP], e_off[EMIT_CAP];
  int32_t* meta = st.meta + (size_t)slot * META_WORDS;
  const int c0 = meta[META_CHUNK_START];
  const int ns = min(D.n_sink, c0), ws = max(ns, c0 - D.window);
  const int32_t* sstart = st.span_start + (size_t)slot * D.max_spans;
  const int32_t* slen = st.span_len + (size_t)slot * D.max_spans;
  int32_t* sel = st.sel_ids + (size_t)slot * D.sel_cap;
  int32_t* list = st.tok_list + (size_t)slot * D.list_cap;
  // host-offloaded KV: the same list as rows of the device pool (initial tokens in place, retrieved token j at
  // stage0 + j, window tokens in the ring), which is what the attention walks
  int32_t* rows = D.offload ? st.row_list + (size_t)slot * D.list_cap : nullptr;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { s_base_cnt = 0; s_base_tok = 0; }
  for (int t = tid; t < ns; t += blockDim.x) { list[t] = t; if (rows) rows[t] = t; }
  __syncthreads();
  for (int i0 = 0; i0 < n; i0 += blockDim.x) {
    const int i = i0 + tid;
    const bool f = i < n && ((selmask[i >> 5] >> (i & 31)) & 1u);
    int a = 0, b = 0;
    if (f) {
      int start, len;
      item_range(D, sstart, slen, c0 + meta[META_CHUNK_LEN], i, start, len);
      clip_span(D, c0, start, len, a, b);
    }
    const int w = f ? max(b - a, 0) : 0;
    // wave-level inclusive scans of (flag, tokens)
    int cs = f ? 1 : 0, ts = w;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int c2 = __shfl_up(cs, o, 64), t2 = __shfl_up(ts, o, 64);
      if (lane >= o) { cs += c2; ts += t2; }
    }
    if (lane == 63) { s_wcnt[wave] = cs; s_wtok[wave] = ts; }
    __syncthreads();
    int coff = s_base_cnt, toff = s_base_tok;
    for (int w2 = 0; w2 < wave; ++w2) { coff += s_wcnt[w2]; toff += s_wtok[w2]; }
    if (f) {
      const int pos = coff + cs - 1;
      if (pos < D.sel_cap) {
        sel[pos] = i;
        if (ids_out) ids_out[pos] = i;
      }
      const int o = ns + toff + ts - w;
      if (pos < EMIT_CAP) {
        e_a[pos] = a; e_len[pos] = w; e_off[pos] = o;
      } else {
        for (int t = 0; t < w; ++t)
          if (o + t < D.list_cap) list[o + t] = a + t;
      }
    }
    __syncthreads();
    if (tid == 0) {
      int c = 0, t = 0;
      for (int w2 = 0; w2 < 16; ++w2) { c += s_wcnt[w2]; t += s_wtok[w2]; }
      s_base_cnt += c; s_base_tok += t;
    }
    __syncthreads();
  }
  const int n_sel = s_base_cnt, n_ret = s_base_tok;
  const int n_win = c0 - ws;
  const int len = ns + n_ret + n_win;
  const bool fits = n_sel <= D.sel_cap && len <= D.list_cap;
  // tokens of the recorded spans: one wavefront per span, lanes along the span
  for (int k = wave; k < min(n_sel, EMIT_CAP); k += 16) {
    const int a = e_a[k], w = e_len[k], o = e_off[k];
    for (int t = lane; t < w; t += 64)
      if (o + t < D.list_cap) list[o + t] = a + t;
  }
  if (fits) {
    for (int t = tid; t < n_win; t += blockDim.x) {
      list[ns + n_ret + t] = ws + t;
      if (rows) rows[ns + n_ret + t] = window_tok_row(D, ws + t);
    }
    if (rows)
      for (int t = tid; t < n_ret; t += blockDim.x) rows[ns + t] = D.stage0 + t;
    // padding: a valid token, masked by position. One tile more than the list's own last tile, because the
    // attention over the retrieved slice alone starts its tiles at the end of the initial tokens.
    const int padded = min(D.list_cap, (len + ATT_BN - 1) / ATT_BN * ATT_BN + ATT_BN);
    for (int t = len + tid; t < padded; t += blockDim.x) { list[t] = 0; if (rows) rows[t] = 0; }
  }
  if (tid == 0) {
    if (!fits) atomicCAS(&st.err[0], 0, LTRI_ECAPACITY);
    meta[META_SEL_CNT] = fits ? n_sel : 0;
    meta[META_LIST_LEN] = fits ? len : 0;
    if (cnt_out) *cnt_out = fits ? n_sel : 0;
  }
}

// ---- top spans under the count cap and the token budget ----
constexpr int SEL_MAX_SPANS = 65536;

// Order key of a span: smaller key = earlier in the order (-score, id). The score's bit pattern
// is mapped to an unsigned integer that grows with the score, then complemented.
__device__ __forceinline__ uint64_t score_key(double s) {
  const uint64_t u = (uint64_t)__double_as_longlong(s + 0.0);          // -0.0 -> +0.0: they compare equal
  const uint64_t up = (u >> 63) ? ~u : (u | 0x8000000000000000ull);   // monotone in s
  return ~up;
}

// Budgeted top-k (Eq. 9 at span granularity): a span is selected iff it is eligible (its clipped
// part is non-empty) and, in the order (score descending, id ascending) over the eligible spans,
// its rank is below k_max and the clipped tokens up to and including it fit the budget. Clipped
// lengths are positive, so this is exactly the longest prefix of that order that fits.
// Rank and cumulated tokens come from all pairs: 32 spans per workgroup, eight threads per span,
// each over an eighth of the other spans (staged through LDS 1024 at a time). A span j comes
// before span i iff key_j < key_i, or the keys are equal and j < i.
constexpr int SEL_SPANS_PER_BLOCK = 32;
constexpr int SEL_PARTS = 256 / SEL_SPANS_PER_BLOCK;      // threads per span
constexpr int SEL_STAGE = 1024;                           // spans staged in LDS at a time
__global__ __launch_bounds__(256) void select_rank_kernel(RetArgs a) {
  __shared__ uint64_t t_key[SEL_STAGE];
  __shared__ int t_clip[SEL_STAGE];
  const Dims& D = a.D;
  const int p = blockIdx.y, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int n = meta[META_N_SPANS], c0 = meta[META_CHUNK_START];
  if ((int)blockIdx.x * SEL_SPANS_PER_BLOCK >= n) return;              // uniform
  const double* scores = a.st.scores + (size_t)slot * D.max_spans;
  const int32_t* sstart = a.st.span_start + (size_t)slot * D.max_spans;
  const int32_t* slen = a.st.span_len + (size_t)slot * D.max_spans;
  const int tid = threadIdx.x, jp = tid % SEL_PARTS;
  const int i = blockIdx.x * SEL_SPANS_PER_BLOCK + tid / SEL_PARTS;
  uint64_t ki = 0;
  int ci = 0;
  if (i < n) {
    int lo, hi;
    clip_span(D, c0, sstart[i], slen[i], lo, hi);
    ci = max(hi - lo, 0);
    ki = score_key(scores[i]);
  }
  int rank = 0, cum = 0;
  for (int j0 = 0; j0 < n; j0 += SEL_STAGE) {
    __syncthreads();
    for (int q = tid; q < SEL_STAGE && j0 + q < n; q += blockDim.x) {
      int lo, hi;
      clip_span(D, c0, sstart[j0 + q], slen[j0 + q], lo, hi);
      t_clip[q] = max(hi - lo, 0);
      t_key[q] = score_key(scores[j0 + q]);
    }
    __syncthreads();
    const int m = min(SEL_STAGE, n - j0);
    for (int jj = jp; jj < m; jj += SEL_PARTS) {
      const int cj = t_clip[jj];
      const uint64_t kj = t_key[jj];
      const bool before = (kj < ki) | ((kj == ki) & (j0 + jj < i));
      rank += (before & (cj > 0)) ? 1 : 0;
      cum += before ? cj : 0;
    }
  }
#pragma unroll
  for (int o = 1; o < SEL_PARTS; o <<= 1) {
    rank += __shfl_xor(rank, o, 64);
    cum += __shfl_xor(cum, o, 64);
  }
  cum += ci;
  if (jp == 0 && i < n) {
    const bool sel = ci > 0 && (D.k_max == 0 || rank < D.k_max) && (D.budget == 0 || (long long)cum <= D.budget);
    a.sc.selflag[(size_t)p * D.max_spans + i] = sel ? 1 : 0;
  }
}

// Selected ids in ascending order, their count, and the context token list (one workgroup per
// KV head).
__global__ __launch_bounds__(1024) void select_emit_kernel(RetArgs a) {
  __shared__ uint32_t selmask[SEL_MAX_SPANS / 32];
  const Dims& D = a.D;
  const int p = blockIdx.x, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int n = meta[META_N_SPANS];
  const uint8_t* flag = a.sc.selflag + (size_t)p * D.max_spans;
  for (int i0 = 0; i0 < n; i0 += blockDim.x) {
    const int i = i0 + threadIdx.x;
    const uint64_t m = __ballot(i < n && flag[i]);
    if ((threadIdx.x & 63) == 0 && i < ((n + 63) & ~63)) {
      selmask[i >> 5] = (uint32_t)m;
      selmask[(i >> 5) + 1] = (uint32_t)(m >> 32);
    }
  }
  __syncthreads();
  int32_t* ids_out = a.sel_ids_out ? a.sel_ids_out + (size_t)p * D.sel_cap : nullptr;
  int32_t* cnt_out = a.sel_cnt_out ? a.sel_cnt_out + p : nullptr;
  emit_selection(D, a.st, slot, selmask, n, ids_out, cnt_out);
}

// ---- step 2 for a one-token chunk (decode) in one launch: one workgroup per (sequence, KV head) ----
// The chunk is its own single query span, so Q^R is the group-summed query row rounded to the
// stored precision. Scores as in score_kernel. The selection rule is the one of select_rank_kernel,
// reached by sorting: eligible spans are sorted by (key, id) in LDS (bitonic network over the next
// power of two), their clipped lengths are scanned in that order, and the selected set is the
// prefix that fits. Spans: at most RT1_MAX_SPANS (the launcher checks its bound).
constexpr int RT1_MAX_SPANS = 8192;
constexpr uint32_t RT1_PAD = 0xffffffffu;
__host__ __device__ constexpr int rt1_pow2(int n) { int m = 64; while (m < n) m <<= 1; return m; }
// dynamic LDS: keys, ids, clipped lengths
__host__ __device__ constexpr size_t rt1_lds_bytes(int bound) { return (size_t)rt1_pow2(bound) * 12 + (size_t)bound * 4; }

// The selection rule by sorting (one workgroup of 1024 threads): skey / sidx[0..npow) hold the order
// keys and ids of the eligible items (the others and the padding: key ~0, id RT1_PAD), clip[id]
// their clipped lengths; npow is a power of two. Items are sorted by (key, id), the clipped
// lengths are scanned in that order, and the longest prefix within k_max items and the token
// budget is marked in selmask (zeroed by the caller). wave_tot: 16 words of LDS.
__device__ __forceinline__ void select_sorted_prefix(const Dims& D, uint64_t* skey, uint32_t* sidx, const int* clip, int npow,
                                     uint32_t* selmask, long long* wave_tot) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // bitonic network, ascending in (key, id)
  if (npow <= (int)blockDim.x) {
    // one position per thread, held in registers; partners at distance < 64 are reached by lane
    // exchanges on the vector ALU, the others through LDS
    const bool live = tid < npow;
    uint64_t key = live ? skey[tid] : ~0ull;
    uint32_t id = live ? sidx[tid] : RT1_PAD;
    // (key, id) pairs are distinct apart from the padding, whose copies are interchangeable
    auto merge = [&](int k, int j, uint64_t pk, uint32_t pid) {
      const bool keep_less = ((tid & j) == 0) == ((tid & k) == 0);
      const bool take = key_less(pk, pid, key, id) == keep_less;
      key = take ? pk : key;
      id = take ? pid : id;
    };
    auto lanes = [&](int k, auto jc) {
      constexpr int J = decltype(jc)::value;
      const uint32_t lo = lane_xor_c<J>((uint32_t)key), hi = lane_xor_c<J>((uint32_t)(key >> 32));
      merge(k, J, ((uint64_t)hi << 32) | lo, lane_xor_c<J>(id));
    };
    using std::integral_constant;
    for (int k = 2; k <= npow; k <<= 1) {
      for (int j = k >> 1; j >= 64; j >>= 1) {
        __syncthreads();
        if (live) { skey[tid] = key; sidx[tid] = id; }
        __syncthreads();
        if (live) merge(k, j, skey[tid ^ j], sidx[tid ^ j]);
      }
      if (k >= 64) lanes(k, integral_constant<int, 32>{});
      if (k >= 32) lanes(k, integral_constant<int, 16>{});
      if (k >= 16) lanes(k, integral_constant<int, 8>{});
      if (k >= 8) lanes(k, integral_constant<int, 4>{});
      if (k >= 4) lanes(k, integral_constant<int, 2>{});
      lanes(k, integral_constant<int, 1>{});
    }
    __syncthreads();
    if (live) { skey[tid] = key; sidx[tid] = id; }
    __syncthreads();
  } else {
    for (int k = 2; k <= npow; k <<= 1) {
      for (int j = k >> 1; j > 0; j >>= 1) {
        for (int t = tid; t < npow / 2; t += blockDim.x) {
          const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;
          const uint64_t ka = skey[lo], kb = skey[hi];
          const uint32_t ia = sidx[lo], ib = sidx[hi];
          const bool a_after_b = (ka > kb) | ((ka == kb) & (ia > ib));
          if (a_after_b == ((lo & k) == 0)) {
            skey[lo] = kb; skey[hi] = ka;
            sidx[lo] = ib; sidx[hi] = ia;
          }
        }
        __syncthreads();
      }
    }
  }
  // clipped tokens up to and including each position of the order; the prefix that fits is selected
  const int E = max(npow / (int)blockDim.x, 1);           // consecutive positions per thread
  long long mine = 0;
  for (int e = 0; e < E; ++e) {
    const int r = tid * E + e;
    const uint32_t id = r < npow ? sidx[r] : RT1_PAD;
    mine += id != RT1_PAD ? clip[id] : 0;
  }
  long long incl = mine;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const long long v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  long long cum = incl - mine;
  for (int w2 = 0; w2 < wave; ++w2) cum += wave_tot[w2];
  for (int e = 0; e < E; ++e) {
    const int r = tid * E + e;
    const uint32_t id = r < npow ? sidx[r] : RT1_PAD;
    if (id != RT1_PAD) {
      cum += clip[id];
      const bool sel = (D.k_max == 0 || r < D.k_max) && (D.budget == 0 || cum <= D.budget);
      if (sel) atomicOr(&selmask[id >> 5], 1u << (id & 31));
    }
  }
}

template <int DT>
__global__ __launch_bounds__(1024) void retrieve_one_token_kernel(RetArgs a, int bound) {
  typedef typename Elt<DT>::type T;
  constexpr int N = 16 / (int)sizeof(T);                // elements per 16-byte piece
  extern __shared__ __attribute__((aligned(16))) unsigned char rt1_lds[];
  __shared__ double qv[128];
  __shared__ uint32_t selmask[RT1_MAX_SPANS / 32 + 2];
  __shared__ long long wave_tot[16];
  const Dims& D = a.D;
  const int p = blockIdx.x, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int d = D.d, tid = threadIdx.x;
  int n = meta[META_N_SPANS], c0 = meta[META_CHUNK_START];
  // Step 1 of a one-token chunk, if asked for: the token is appended as a span of one, its key is the
  // stored vector (what append_single_kernel does). The table entry written here is read back below by
  // other threads of this workgroup, so a barrier stands on either side of the writes.
  if (a.append_first) {
    const int base = n;
    c0 = a.bp.c0[bi];
    const bool fits = base + 1 <= D.max_spans;
    __syncthreads();                                    // every thread has read the old count
    if (fits && tid < d) {
      const T* row = reinterpret_cast<const T*>(a.k_arena) + arena_off(D, slot) + (size_t)chunk_tok_row(D, c0, c0) * d;
      (reinterpret_cast<T*>(a.st.krep) + ((size_t)slot * D.max_spans + base) * d)[tid] = row[tid];
    }
    if (tid == 0) {
      if (fits) {
        a.st.span_start[(size_t)slot * D.max_spans + base] = c0;
        a.st.span_len[(size_t)slot * D.max_spans + base] = 1;
      } else {
        atomicCAS(&a.st.err[0], 0, LTRI_ECAPACITY);
      }
      meta[META_N_SPANS] = fits ? base + 1 : base;
      meta[META_CHUNK_FIRST] = base;
      meta[META_CHUNK_NSP] = fits ? 1 : 0;
      meta[META_CHUNK_START] = c0;
      meta[META_CHUNK_LEN] = 1;
    }
    n = fits ? base + 1 : base;
    __threadfence_block();
    __syncthreads();
  }
  n = min(n, bound);
  const int npow = rt1_pow2(n);
  uint64_t* skey = reinterpret_cast<uint64_t*>(rt1_lds);
  uint32_t* sidx = reinterpret_cast<uint32_t*>(rt1_lds + (size_t)rt1_pow2(bound) * 8);
  int* clip = reinterpret_cast<int*>(rt1_lds + (size_t)rt1_pow2(bound) * 12);
  // scores, order keys and clipped lengths: four lanes per span
  const T* krep = reinterpret_cast<const T*>(a.st.krep) + (size_t)slot * D.max_spans * d;
  double* scores = a.st.scores + (size_t)slot * D.max_spans;
  const int32_t* sstart = a.st.span_start + (size_t)slot * D.max_spans;
  const int32_t* slen = a.st.span_len + (size_t)slot * D.max_spans;
  constexpr int PPL = 128 / N / 4;                      // 16-byte pieces per lane (d = 128)
  constexpr int PASSES = DT == LTRI_BF16 ? 3 : 1;       // spans per thread whose loads are in flight together
  const int part = tid & 3;
  uint4 kv[PASSES][PPL];
  int ss[PASSES], sl[PASSES];                           // the spans' extents travel with their keys
  auto load_batch = [&](int i00) {
#pragma unroll
    for (int u = 0; u < PASSES; ++u) {
      const int ic = max(min(i00 + 256 * u + (tid >> 2), n - 1), 0);
      const uint4* krow = reinterpret_cast<const uint4*>(krep + (size_t)ic * d);
#pragma unroll
      for (int q = 0; q < PPL; ++q) kv[u][q] = krow[part + 4 * q];
      ss[u] = sstart[ic];
      sl[u] = slen[ic];
    }
  };
  load_batch(0);                                        // in flight while the query row is fetched
  // Q^R of the chunk's one span
  if (tid < d) {
    const T* Qb = reinterpret_cast<const T*>(a.q) + (size_t)bi * D.Hq * d + (size_t)h * D.G * d;
    double sum = 0.0;
    for (int g = 0; g < D.G; ++g) sum += Elt<DT>::to_f64(Qb[(size_t)g * d + tid]);
    const T r = Elt<DT>::from_f64(sum);
    reinterpret_cast<T*>(a.sc.qrep)[(size_t)p * a.Lp * d + tid] = r;
    qv[tid] = Elt<DT>::to_f64(r);
  }
  for (int w = tid; w < (n + 31) / 32 + 2; w += blockDim.x) selmask[w] = 0u;
  __syncthreads();
  for (int i00 = 0; i00 < npow; i00 += 256 * PASSES) {
    if (i00 > 0) load_batch(i00);
#pragma unroll
    for (int u = 0; u < PASSES; ++u) {
      const int i = i00 + 256 * u + (tid >> 2);
      double acc = 0.0;
#pragma unroll
      for (int q = 0; q < PPL; ++q) {
        const int pc = part + 4 * q;
        double k[8];
        if constexpr (DT == LTRI_BF16) {
          const uint32_t w[4] = {kv[u][q].x, kv[u][q].y, kv[u][q].z, kv[u][q].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            k[2 * e] = (double)__uint_as_float(w[e] << 16);
            k[2 * e + 1] = (double)__uint_as_float(w[e] & 0xffff0000u);
          }
        } else {
          k[0] = (double)__uint_as_float(kv[u][q].x); k[1] = (double)__uint_as_float(kv[u][q].y);
          k[2] = (double)__uint_as_float(kv[u][q].z); k[3] = (double)__uint_as_float(kv[u][q].w);
        }
#pragma unroll
        for (int e = 0; e < N; ++e) acc = fma(k[e], qv[pc * N + e], acc);
      }
      acc += __shfl_xor(acc, 1, 64);
      acc += __shfl_xor(acc, 2, 64);
      if (part == 0 && i < npow) {
        int c = 0;
        if (i < n) {
          int lo, hi;
          clip_span(D, c0, ss[u], sl[u], lo, hi);
          c = max(hi - lo, 0);
          scores[i] = acc;
          clip[i] = c;
        }
        // spans that cannot be retrieved go to the end of the order with the padding
        skey[i] = c > 0 ? score_key(acc) : ~0ull;
        sidx[i] = c > 0 ? (uint32_t)i : RT1_PAD;
      }
    }
  }
  __syncthreads();
  select_sorted_prefix(D, skey, sidx, clip, npow, selmask, wave_tot);
  __syncthreads();
  int32_t* ids_out = a.sel_ids_out ? a.sel_ids_out + (size_t)p * D.sel_cap : nullptr;
  int32_t* cnt_out = a.sel_cnt_out ? a.sel_cnt_out + p : nullptr;
  emit_selection(D, a.st, slot, selmask, n, ids_out, cnt_out);
}

// ---- step 2 of a long chunk in one launch: the scores of all stored spans (Eq. 8, maximum over the query spans as
//      in Eq. 9), the budgeted selection by sorting and the lists. gridDim.x = (sequence, KV head) problems;
//      the gridDim.y workgroups of a problem share its scoring, 256 spans at a time each, so that the stored vectors
//      stream in through many compute units, and the one that finishes last (a ticket counter, left at zero again)
//      sorts and writes the lists. Q^R is either in place (qrep_partial_kernel) or, with qrep_from_sums, built
//      here from the running sums of the chunk's query rows, two rows per query span, and so are, with rs.k_arena, the
//      mean keys of the chunk's own spans (Sec. 3.3.1): every workgroup of a problem writes the same values to
//      the same places and reads its own copy back after a barrier. head_dim 128, spans retrieved (not units), at
//      most RT1_MAX_SPANS stored spans (the launcher checks). ----
template <int DT>
__global__ __launch_bounds__(1024) void retrieve_chunk_kernel(RetArgs a, int bound) {
  typedef typename Elt<DT>::type T;
  extern __shared__ __attribute__((aligned(16))) unsigned char rt1_lds[];
  __shared__ uint32_t selmask[RT1_MAX_SPANS / 32 + 2];
  __shared__ long long wave_tot[16];
  __shared__ int s_last;
  const Dims& D = a.D;
  const int pl = blockIdx.x, bi = a.batch_off + pl / D.Hkv, h = pl % D.Hkv, pg = bi * D.Hkv + h;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int d = 128, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = min(meta[META_N_SPANS], bound), c0 = meta[META_CHUNK_START];
  const int nqs = meta[META_CHUNK_NSP], first = meta[META_CHUNK_FIRST];
  const int32_t* sstart = a.st.span_start + (size_t)slot * D.max_spans;
  const int32_t* slen = a.st.span_len + (size_t)slot * D.max_spans;
  T* qrep = reinterpret_cast<T*>(a.sc.qrep) + (size_t)pg * a.Lp * d;
  T* krep_w = reinterpret_cast<T*>(a.st.krep) + (size_t)slot * D.max_spans * d;
  if (a.qrep_from_sums && 256 * (int)blockIdx.y < n) {      // (a workgroup without spans to score needs none of it)
    // representative = (running sum at the span's end - running sum at its start) / length, rounded to the dtype
    const int n_q = a.rs.n_q, nblk = (n_q + RUNSUM_BLOCK - 1) / RUNSUM_BLOCK;
    double* carry = reinterpret_cast<double*>(rt1_lds);   // [2][blocks][128]: sum of the rows of all earlier blocks
    const double* qpre = a.rs.out + (size_t)pl * a.rs.rows * d;
    const double* kpre = qpre + a.rs.keys_off;
    const bool with_keys = a.rs.k_arena != nullptr;
    if (tid < 2 * d && (tid < d || with_keys)) {
      const int c = tid & 127;
      const double* src = tid < d ? qpre : kpre;
      double* dst = carry + (tid < d ? 0 : nblk * d);
      double run = 0.0;
      for (int b0 = 0; b0 < nblk; b0 += 16) {
        double v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u)
          v[u] = src[(size_t)min((b0 + u) * RUNSUM_BLOCK + RUNSUM_BLOCK - 1, n_q - 1) * d + c];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          if (b0 + u < nblk) dst[(b0 + u) * d + c] = run;
          run += v[u];
        }
      }
    }
    __syncthreads();
    const int c = tid & 127;
    for (int q = tid >> 7; q < nqs; q += 8) {
      const int len = slen[first + q];
      const int x0 = min(max(sstart[first + q] - c0, 0), n_q), x1 = min(x0 + len, n_q);
      const int b0 = (max(x0, 1) - 1) / RUNSUM_BLOCK, b1 = (max(x1, 1) - 1) / RUNSUM_BLOCK;
      const size_t o0 = (size_t)(max(x0, 1) - 1) * d + c, o1 = (size_t)(max(x1, 1) - 1) * d + c;
      const double q0 = x0 > 0 ? carry[b0 * d + c] + qpre[o0] : 0.0;
      const double q1 = x1 > 0 ? carry[b1 * d + c] + qpre[o1] : 0.0;
      qrep[(size_t)q * d + c] = Elt<DT>::from_f64((q1 - q0) / (double)len);
      if (with_keys) {
        const double k0 = x0 > 0 ? carry[(nblk + b0) * d + c] + kpre[o0] : 0.0;
        const double k1 = x1 > 0 ? carry[(nblk + b1) * d + c] + kpre[o1] : 0.0;
        krep_w[(size_t)(first + q) * d + c] = Elt<DT>::from_f64((k1 - k0) / (double)len);
      }
    }
    __syncthreads();
  }
  const int n_score = (int)gridDim.y;
  const T* krep = reinterpret_cast<const T*>(a.st.krep) + (size_t)slot * D.max_spans * d;
  double* scores = a.st.scores + (size_t)slot * D.max_spans;
  for (int i0 = 256 * (int)blockIdx.y + 16 * wave; i0 < n; i0 += 256 * n_score) {   // a tile of 16 spans per wavefront
    double best[4];
    score_tile_f64<DT>(krep, n, i0, qrep, nqs, d, best);
    if ((lane & 15) == 0) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int i = i0 + 4 * v + (lane >> 4);
        // stored and (below) loaded at device scope, as the pieces of Q^R are in qrep_partial_kernel
        if (i < n) __hip_atomic_store(scores + i, best[v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  __syncthreads();                                        // the workgroup's stores have completed
  if (n_score > 1) {
    if (tid == 0) s_last = atomicAdd(&a.sc.tickets[a.ticket_base + pl], 1) == n_score - 1;
    __syncthreads();
    if (!s_last) return;
    if (tid == 0) a.sc.tickets[a.ticket_base + pl] = 0;
  }
  const int npow = rt1_pow2(n);
  uint64_t* skey = reinterpret_cast<uint64_t*>(rt1_lds);
  uint32_t* sidx = reinterpret_cast<uint32_t*>(rt1_lds + (size_t)rt1_pow2(bound) * 8);
  int* clip = reinterpret_cast<int*>(rt1_lds + (size_t)rt1_pow2(bound) * 12);
  for (int w = tid; w < (n + 31) / 32 + 2; w += blockDim.x) selmask[w] = 0u;
  for (int i = tid; i < npow; i += blockDim.x) {
    int c = 0;
    double sc = 0.0;
    if (i < n) {
      int lo, hi;
      clip_span(D, c0, sstart[i], slen[i], lo, hi);
      c = max(hi - lo, 0);
      sc = __hip_atomic_load(scores + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      clip[i] = c;
    }
    // spans that cannot be retrieved go to the end of the order with the padding
    skey[i] = c > 0 ? score_key(sc) : ~0ull;
    sidx[i] = c > 0 ? (uint32_t)i : RT1_PAD;
  }
  __syncthreads();
  select_sorted_prefix(D, skey, sidx, clip, npow, selmask, wave_tot);
  __syncthreads();
  int32_t* ids_out = a.sel_ids_out ? a.sel_ids_out + (size_t)pg * D.sel_cap : nullptr;
  int32_t* cnt_out = a.sel_cnt_out ? a.sel_cnt_out + pg : nullptr;
  emit_selection(D, a.st, slot, selmask, n, ids_out, cnt_out);
}

// ---- retrieval by memory units (Eq. 9 as written): a unit scores the maximum over its spans; the
//      top units within k_max and the token budget are retrieved whole. One workgroup per
//      (sequence, KV head); the spans' scores are already in place. ----
__global__ __launch_bounds__(1024) void unit_select_kernel(RetArgs a, int unit_bound) {
  extern __shared__ __attribute__((aligned(16))) unsigned char rt1_lds[];
  __shared__ uint32_t selmask[RT1_MAX_SPANS / 32 + 2];
  __shared__ long long wave_tot[16];
  const Dims& D = a.D;
  const int p = blockIdx.x, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int n_spans = meta[META_N_SPANS], c0 = meta[META_CHUNK_START];
  const int n_tokens = c0 + meta[META_CHUNK_LEN];
  const int n = min(item_count(D, meta), unit_bound);
  const int npow = rt1_pow2(n), tid = threadIdx.x;
  uint64_t* skey = reinterpret_cast<uint64_t*>(rt1_lds);
  uint32_t* sidx = reinterpret_cast<uint32_t*>(rt1_lds + (size_t)rt1_pow2(unit_bound) * 8);
  int* clip = reinterpret_cast<int*>(rt1_lds + (size_t)rt1_pow2(unit_bound) * 12);
  const double* scores = a.st.scores + (size_t)slot * D.max_spans;
  const int32_t* sstart = a.st.span_start + (size_t)slot * D.max_spans;
  for (int w = tid; w < (n + 31) / 32 + 2; w += blockDim.x) selmask[w] = 0u;
  for (int u = tid; u < npow; u += blockDim.x) {
    int c = 0;
    double best = -INFINITY;
    if (u < n) {
      int lo, hi;
      clip_span(D, c0, u * D.unit, min(D.unit, n_tokens - u * D.unit), lo, hi);
      c = max(hi - lo, 0);
      if (c > 0) {
        // spans are stored in stream order: the unit's spans start in [u unit, (u + 1) unit)
        int first = 0, last = n_spans;
        while (first < last) { const int mid = (first + last) >> 1; if (sstart[mid] < u * D.unit) first = mid + 1; else last = mid; }
        for (int i = first; i < n_spans && sstart[i] < (u + 1) * D.unit; ++i) best = fmax(best, scores[i]);
      }
      clip[u] = c;
    }
    skey[u] = c > 0 ? score_key(best) : ~0ull;
    sidx[u] = c > 0 ? (uint32_t)u : RT1_PAD;
  }
  __syncthreads();
  select_sorted_prefix(D, skey, sidx, clip, npow, selmask, wave_tot);
  __syncthreads();
  int32_t* ids_out = a.sel_ids_out ? a.sel_ids_out + (size_t)p * D.sel_cap : nullptr;
  int32_t* cnt_out = a.sel_cnt_out ? a.sel_cnt_out + p : nullptr;
  emit_selection(D, a.st, slot, selmask, n, ids_out, cnt_out);
}

// ---- collaborative voting over memory units (Sec. 3.5): the layer selects on its own, then the
//      units are re-ordered by the weighted votes of the earlier layers' selections and its own
//      (votes descending, own score descending, id ascending) and the prefix that fits is kept ----
__device__ __forceinline__ uint32_t float_key_desc(float v) {          // smaller key = larger value
  const uint32_t u = __float_as_uint(v + 0.0f);
  return ~((u >> 31) ? ~u : (u | 0x80000000u));
}

__global__ __launch_bounds__(1024) void unit_vote_select_kernel(RetArgs a, int unit_bound, VoteArgs v) {
  extern __shared__ __attribute__((aligned(16))) unsigned char rt1_lds[];
  __shared__ uint32_t selmask[RT1_MAX_SPANS / 32 + 2], ownmask[RT1_MAX_SPANS / 32 + 2];
  __shared__ long long wave_tot[16];
  const Dims& D = a.D;
  const int p = blockIdx.x, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int seq = a.bp.seq[bi];
  const int slot = slot_of(D, a.layer, seq, h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int n_spans = meta[META_N_SPANS], c0 = meta[META_CHUNK_START];
  const int n_tokens = c0 + meta[META_CHUNK_LEN];
  const int n = min(item_count(D, meta), unit_bound);
  const int npow = rt1_pow2(n), tid = threadIdx.x;
  const size_t pw = (size_t)rt1_pow2(unit_bound);
  uint64_t* skey = reinterpret_cast<uint64_t*>(rt1_lds);
  uint32_t* sidx = reinterpret_cast<uint32_t*>(rt1_lds + pw * 8);
  int* clip = reinterpret_cast<int*>(rt1_lds + pw * 12);
  int* rank = clip + unit_bound;
  float* vote = reinterpret_cast<float*>(rank + unit_bound);
  const double* scores = a.st.scores + (size_t)slot * D.max_spans;
  const int32_t* sstart = a.st.span_start + (size_t)slot * D.max_spans;
  for (int w = tid; w < (n + 31) / 32 + 2; w += blockDim.x) { selmask[w] = 0u; ownmask[w] = 0u; }
  for (int u = tid; u < npow; u += blockDim.x) {
    int c = 0;
    double best = -INFINITY;
    if (u < n) {
      int lo, hi;
      clip_span(D, c0, u * D.unit, min(D.unit, n_tokens - u * D.unit), lo, hi);
      c = max(hi - lo, 0);
      if (c > 0) {
        int first = 0, last = n_spans;
        while (first < last) { const int mid = (first + last) >> 1; if (sstart[mid] < u * D.unit) first = mid + 1; else last = mid; }
        for (int i = first; i < n_spans && sstart[i] < (u + 1) * D.unit; ++i) best = fmax(best, scores[i]);
      }
      clip[u] = c;
      vote[u] = 0.f;
      rank[u] = 0;
    }
    skey[u] = c > 0 ? score_key(best) : ~0ull;
    sidx[u] = c > 0 ? (uint32_t)u : RT1_PAD;
  }
  __syncthreads();
  select_sorted_prefix(D, skey, sidx, clip, npow, ownmask, wave_tot);      // the layer's own selection
  __syncthreads();
  for (int r = tid; r < npow; r += blockDim.x)
    if (sidx[r] != RT1_PAD) rank[sidx[r]] = r;                            // position in the order of the own scores
  // votes, one voter after the other (float32 sums in a fixed order); a voter lists a unit at most once
  for (int k = 0; k < v.n_voters; ++k) {
    const int vslot = slot_of(D, v.layer[k], seq, h);
    const int cnt = min(a.st.meta[(size_t)vslot * META_WORDS + META_SEL_CNT], D.sel_cap);
    const int32_t* ids = a.st.sel_ids + (size_t)vslot * D.sel_cap;
    for (int j = tid; j < cnt; j += blockDim.x) {
      const int u = ids[j];
      if (u >= 0 && u < n) vote[u] += v.weight[k];
    }
    __syncthreads();
  }
  for (int u = tid; u < n; u += blockDim.x)
    if ((ownmask[u >> 5] >> (u & 31)) & 1u) vote[u] += v.own_weight;
  __syncthreads();
  for (int u = tid; u < npow; u += blockDim.x) {
    const bool ok = u < n && clip[u] > 0;
    skey[u] = ok ? (((uint64_t)float_key_desc(vote[u]) << 32) | (uint32_t)rank[u]) : ~0ull;
    sidx[u] = ok ? (uint32_t)u : RT1_PAD;
  }
  __syncthreads();
  select_sorted_prefix(D, skey, sidx, clip, npow, selmask, wave_tot);
  __syncthreads();
  int32_t* ids_out = a.sel_ids_out ? a.sel_ids_out + (size_t)p * D.sel_cap : nullptr;
  int32_t* cnt_out = a.sel_cnt_out ? a.sel_cnt_out + p : nullptr;
  emit_selection(D, a.st, slot, selmask, n, ids_out, cnt_out);
}

// ---- caller-forced selection: ids already copied (ascending, unique) into sel_ids ----
struct ForceArgs { Dims D; DevState st; int layer, seq, h, n_ids; };

__global__ __launch_bounds__(1024) void force_list_kernel(ForceArgs a) {
  __shared__ uint32_t selmask[SEL_MAX_SPANS / 32];
  const Dims& D = a.D;
  const int slot = slot_of(D, a.layer, a.seq, a.h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int c0 = meta[META_CHUNK_START];
  const int n = item_count(D, meta);
  const int tid = threadIdx.x;
  for (int w = tid; w < (n + 31) / 32; w += blockDim.x) selmask[w] = 0u;
  __syncthreads();
  const int32_t* ids = a.st.sel_ids + (size_t)slot * D.sel_cap;
  for (int k = tid; k < a.n_ids; k += blockDim.x) {
    const int i = ids[k];
    if (i >= 0 && i < n) {
      int start, len, lo, hi;
      item_range(D, a.st.span_start + (size_t)slot * D.max_spans, a.st.span_len + (size_t)slot * D.max_spans,
                 c0 + meta[META_CHUNK_LEN], i, start, len);
      clip_span(D, c0, start, len, lo, hi);
      if (hi > lo) atomicOr(&selmask[i >> 5], 1u << (i & 31));
    }
  }
  __syncthreads();
  emit_selection(D, a.st, slot, selmask, n, nullptr, nullptr);
}

bool retrieve_is_one_launch(const Dims& D, int n_q, int span_bound) {
  return n_q == 1 && span_bound >= 1 && span_bound <= RT1_MAX_SPANS && D.d == 128 && D.unit == 0;
}

bool retrieve_reads_running_sums(const Dims& D, int n_q) {
  return n_q > QREP_PIECE && D.d == 128 && D.unit == 0 && D.dtype == LTRI_BF16 && D.rep_mode == LTRI_REP_MEAN &&
         (size_t)n_q * 16 + 2048 <= 116 * 1024;     // the readers' table of block sums shares the LDS of the sort
}

bool retrieve_stores_rep_keys(const Dims& D, int n_q) {
  return n_q > QREP_PIECE && D.rep_mode == LTRI_REP_MEAN;
}

hipError_t launch_retrieve(const Dims& D, const DevState& st, const DevScratch& sc, int sc_max_problems,
                           const void* q, int layer, const BatchPos& bp, int seq_count, int n_q, int span_bound,
                           int32_t* sel_ids_out, int32_t* sel_cnt_out, const VoteArgs* votes, const void* append_k_arena,
                           const void* rep_k_arena, bool sums_ready, hipStream_t s) {
  RetArgs a;
  a.D = D; a.st = st; a.sc = sc; a.q = q; a.layer = layer; a.seq_count = seq_count; a.n_q = n_q;
  a.k_arena = append_k_arena; a.append_first = append_k_arena != nullptr;
  a.rep_k_arena = rep_k_arena;
  a.qrep_by_last = false; a.ticket_base = 0; a.qrep_from_sums = 0;
  a.rs = RunSums{};
  if (rep_k_arena && !retrieve_stores_rep_keys(D, n_q)) return hipErrorInvalidValue;
  if (a.append_first && !retrieve_is_one_launch(D, n_q, span_bound)) return hipErrorInvalidValue;
  a.Lp = (n_q + SEG_TB - 1) / SEG_TB * SEG_TB;
  a.sel_ids_out = sel_ids_out; a.sel_cnt_out = sel_cnt_out; a.bp = bp;
  const int P = seq_count * D.Hkv;
  const bool bf = D.dtype == LTRI_BF16;
  a.batch_off = 0;
  if (retrieve_is_one_launch(D, n_q, span_bound)) {
    // decode: the whole step in one launch
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&retrieve_one_token_kernel<LTRI_BF16>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)rt1_lds_bytes(RT1_MAX_SPANS));
      if (e != hipSuccess) return e;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&retrieve_one_token_kernel<LTRI_F32>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)rt1_lds_bytes(RT1_MAX_SPANS));
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    const size_t lds = rt1_lds_bytes(span_bound);
    if (bf) retrieve_one_token_kernel<LTRI_BF16><<<P, 1024, lds, s>>>(a, span_bound);
    else    retrieve_one_token_kernel<LTRI_F32><<<P, 1024, lds, s>>>(a, span_bound);
    return hipGetLastError();
  }
  a.units_cap = n_q / QREP_PIECE + n_q;                  // pieces of all spans of a chunk, at most
  // Long chunks of 128-wide heads with spans as the retrieval unit: after the pieces' sums everything else of the
  // step is one launch per batch of sequences (retrieve_chunk_kernel).
  // (its sort arrays share the 160 KB of LDS with 42 KB of staging and list scratch)
  const bool one_tail = n_q > QREP_PIECE && D.d == 128 && D.unit == 0 && !votes && span_bound >= 1 &&
                        span_bound <= RT1_MAX_SPANS && rt1_lds_bytes(span_bound) <= 116 * 1024;
  if (one_tail) {
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&retrieve_chunk_kernel<LTRI_BF16>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 116 * 1024);
      if (e != hipSuccess) return e;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&retrieve_chunk_kernel<LTRI_F32>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 116 * 1024);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
  }
  if (n_q > QREP_PIECE) {
    const int per = sc_max_problems / D.Hkv;               // sequences the piece buffer holds
    const int gx = QREP_GRID_X + (rep_k_arena ? QREP_GRID_X : 0);
    // Mean representatives in bf16 (whose sums are exact in fp64): Q^R and the chunk's mean keys come from running
    // sums of the query and key rows, which need no span boundaries (no piece sums, no ticket).
    const bool from_sums = one_tail && retrieve_reads_running_sums(D, n_q);
    size_t lds = rt1_lds_bytes(span_bound);
    if (from_sums) {
      const size_t carry_bytes = (size_t)((n_q + RUNSUM_BLOCK - 1) / RUNSUM_BLOCK) * 2 * 128 * 8;
      if (lds < carry_bytes) lds = carry_bytes;
      a.rs = running_sums_of(D, sc, sc_max_problems, q, rep_k_arena, n_q);
    }
    if (sums_ready && (!from_sums || seq_count > per)) sums_ready = false;     // not usable: taken here
    for (int off = 0; off < seq_count; off += per) {
      const int cnt = seq_count - off < per ? seq_count - off : per;
      a.batch_off = off;
      dim3 gp(gx, cnt * D.Hkv), gf(n_q < 64 ? n_q : 64, cnt * D.Hkv);
      a.qrep_by_last = one_tail;
      a.ticket_base = sc_max_problems;                      // the second half of the counters
      if (from_sums) {
        if (!sums_ready) running_sums_kernel<LTRI_BF16><<<dim3(running_sums_blocks(a.rs, 16), cnt * D.Hkv), 1024, 0, s>>>(a);
        a.qrep_from_sums = 1;
      } else {
        if (bf) qrep_partial_kernel<LTRI_BF16><<<gp, 1024, 0, s>>>(a);
        else    qrep_partial_kernel<LTRI_F32><<<gp, 1024, 0, s>>>(a);
      }
      if (one_tail) {
        const dim3 gt(cnt * D.Hkv, (span_bound + 255) / 256);
        if (bf) retrieve_chunk_kernel<LTRI_BF16><<<gt, 1024, lds, s>>>(a, span_bound);
        else    retrieve_chunk_kernel<LTRI_F32><<<gt, 1024, lds, s>>>(a, span_bound);
      } else {
        if (bf) qrep_final_kernel<LTRI_BF16><<<gf, 128, 0, s>>>(a);
        else    qrep_final_kernel<LTRI_F32><<<gf, 128, 0, s>>>(a);
      }
    }
    a.batch_off = 0;
    if (one_tail) return hipGetLastError();
  } else {
    dim3 gq(n_q < 64 ? n_q : 64, P);
    if (bf) qrep_kernel<LTRI_BF16><<<gq, 1024, 0, s>>>(a);
    else    qrep_kernel<LTRI_F32><<<gq, 1024, 0, s>>>(a);
  }
  int gx = (span_bound + 63) / 64;
  if (gx < 1) gx = 1;
  dim3 gs(gx, P);
  const size_t qs_bytes = (size_t)SCORE_QBATCH * D.d * sizeof(double);
  if (bf) score_kernel<LTRI_BF16><<<gs, 256, qs_bytes, s>>>(a);
  else    score_kernel<LTRI_F32><<<gs, 256, qs_bytes, s>>>(a);
  if (D.unit > 0) {
    const int unit_bound = (int)(D.max_tokens / D.unit) + 1;           // units a full stream has, at most
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&unit_select_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)rt1_lds_bytes(RT1_MAX_SPANS));
      if (e != hipSuccess) return e;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&unit_vote_select_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(rt1_lds_bytes(VOTE_MAX_UNITS) + 8 * VOTE_MAX_UNITS));
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    if (votes && unit_bound > VOTE_MAX_UNITS) return hipErrorInvalidValue;     // the host API checks this first
    if (votes) unit_vote_select_kernel<<<P, 1024, rt1_lds_bytes(unit_bound) + 8 * (size_t)unit_bound, s>>>(a, unit_bound, *votes);
    else       unit_select_kernel<<<P, 1024, rt1_lds_bytes(unit_bound), s>>>(a, unit_bound);
    return hipGetLastError();
  }
  int gr = (span_bound + SEL_SPANS_PER_BLOCK - 1) / SEL_SPANS_PER_BLOCK;
  if (gr < 1) gr = 1;
  select_rank_kernel<<<dim3(gr, P), 256, 0, s>>>(a);
  select_emit_kernel<<<P, 1024, 0, s>>>(a);
  return hipGetLastError();
}

// ---- persistent selection (Sec. 3.5, Persistent Mechanism): the ids selected earlier stay, the
//      token list is rebuilt for the slot's current chunk (the window has moved on) ----
__global__ __launch_bounds__(1024) void persist_list_kernel(RetArgs a) {
  __shared__ uint32_t selmask[SEL_MAX_SPANS / 32];
  const Dims& D = a.D;
  const int p = blockIdx.x, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int c0 = meta[META_CHUNK_START];
  const int n = item_count(D, meta);
  const int cnt = min(meta[META_SEL_CNT], D.sel_cap);
  const int tid = threadIdx.x;
  for (int w = tid; w < (n + 31) / 32; w += blockDim.x) selmask[w] = 0u;
  __syncthreads();
  const int32_t* ids = a.st.sel_ids + (size_t)slot * D.sel_cap;
  for (int k = tid; k < cnt; k += blockDim.x) {
    const int i = ids[k];
    if (i >= 0 && i < n) {
      int start, len, lo, hi;
      item_range(D, a.st.span_start + (size_t)slot * D.max_spans, a.st.span_len + (size_t)slot * D.max_spans,
                 c0 + meta[META_CHUNK_LEN], i, start, len);
      clip_span(D, c0, start, len, lo, hi);
      if (hi > lo) atomicOr(&selmask[i >> 5], 1u << (i & 31));
    }
  }
  __syncthreads();
  emit_selection(D, a.st, slot, selmask, n, nullptr, nullptr);
}

hipError_t launch_persist_list(const Dims& D, const DevState& st, int layer, const BatchPos& bp, int seq_count,
                               hipStream_t s) {
  RetArgs a;
  memset(&a, 0, sizeof a);
  a.D = D; a.st = st; a.layer = layer; a.seq_count = seq_count; a.bp = bp;
  persist_list_kernel<<<seq_count * D.Hkv, 1024, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_force_list(const Dims& D, const DevState& st, int layer, int seq, int kv_head,
                             int n_ids, hipStream_t s) {
  ForceArgs a{D, st, layer, seq, kv_head, n_ids};
  force_list_kernel<<<1, 1024, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace ltri
