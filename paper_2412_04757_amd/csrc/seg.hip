// Step 1 on the device: segmentation of a chunk into spans (Sec. 3.2, Eq. 1-5; appendix
// "NMS Input Filtration"; greedy NMS) and the spans' representative keys (Sec. 3.3.1).
//
// The chunk's L x L causal map M is never written to memory. It is cut into 64 x 64 tiles;
// each tile is computed on the matrix cores from the chunk's K (and Q) rows whenever it is
// needed, which is cheaper than storing L^2 doubles. The Triangle-Attention score (Eq. 4,
// second form)
//     S*[x][y] = sum_{i <= y} sum_{j >= x} M[i][j]
// is a 2-D cumulative sum from the top-right corner. It is assembled per tile (I, J) from
//   - the tile-local corner sum,
//   - a row carry    RC[J][i] = sum of row i over the tiles to the right of J,
//   - a column carry  A[I][x] = sum over all rows above block I of their sum from column x on.
// Pass 1 emits per-tile row sums / suffix-scanned column sums / totals; pass 2 recomputes each tile,
// adds up its two carries from those sums, finishes S = S* - theta * n_h * tri(y - x + 1)
// (Eq. 5) and reduces every anti-diagonal x + y = s inside the tile; pass 3 merges the tile
// results per anti-diagonal, runs the greedy NMS (best live candidate first) and cuts the chunk.
// All sums are fp64 in a fixed order, so the result is deterministic.
#include "device_common.h"
#include <type_traits>
#include "span_mean.h"
#include "running_sums.h"

namespace ltri {

struct SegArgs {
  Dims D; DevState st; DevScratch sc;
  const void* k_arena; const void* q_seg;
  int layer; int batch_off; int n_new; int nb; int Lp; int ntiles;
  BatchPos bp;
  int sum_wgs;     // further workgroups per problem of seg_select_kernel's launch that take running sums for step 2
  RunSums rs;
};

__device__ __forceinline__ void tile_decode(int t, int& I, int& J) {
  int i = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
  while ((i + 1) * (i + 2) / 2 <= t) ++i;
  while (i * (i + 1) / 2 > t) --i;
  I = i; J = t - i * (i + 1) / 2;
}

// Operand staging: 64 rows x 256 bytes (the kc-th 256-byte piece of every row's d-vector) are
// copied global -> LDS with full-row coalescing; inside a row the sixteen 16-byte pieces are
// XOR-permuted with the row number so that the fragment reads below are free of bank conflicts.
template <typename T>
__device__ __forceinline__ void stage_rows(unsigned char* dst, const T* base, size_t row_stride, int row0,
                                           int L, int kc) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int q = threadIdx.x + 256 * i;
    const int row = q >> 4, piece = q & 15;
    const int grow = min(row0 + row, L - 1);                 // clamped; masked by the caller
    const uint4 v = *(reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(base + (size_t)grow * row_stride) + kc * 256) + piece);
    *reinterpret_cast<uint4*>(dst + row * 256 + ((piece ^ (row & 15)) << 4)) = v;
  }
}

// 32 x 32 block of dot products on the matrix cores over one staged 256-byte piece:
// acc[v] += sum_k A[r(v)][k] * B[c][k] with c = lane % 32 and
// r(v) = 8 * (v / 4) + 4 * (lane / 32) + v % 4. abuf / bbuf are the staged 64-row operands,
// arow0 / brow0 the first of the wave's 32 rows in them.
template <int DT> struct TileDot;
template <> struct TileDot<LTRI_BF16> {
  __device__ static __forceinline__ void run(const unsigned char* abuf, const unsigned char* bbuf, int arow0,
                                             int brow0, int l32, int hf, f32x16_t& acc) {
    const unsigned char* ar = abuf + (arow0 + l32) * 256;
    const unsigned char* br = bbuf + (brow0 + l32) * 256;
    const int sw = l32 & 15;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const uint4 av = *reinterpret_cast<const uint4*>(ar + (((2 * kk + hf) ^ sw) << 4));
      const uint4 bv = *reinterpret_cast<const uint4*>(br + (((2 * kk + hf) ^ sw) << 4));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, av),
                                                    __builtin_bit_cast(bf16x8_t, bv), acc, 0, 0, 0);
    }
  }
};
template <> struct TileDot<LTRI_F32> {
  __device__ static __forceinline__ void run(const unsigned char* abuf, const unsigned char* bbuf, int arow0,
                                             int brow0, int l32, int hf, f32x16_t& acc) {
    const unsigned char* ar = abuf + (arow0 + l32) * 256;
    const unsigned char* br = bbuf + (brow0 + l32) * 256;
    const int sw = l32 & 15;
#pragma unroll
    for (int c = 0; c < 16; ++c) {                  // four floats per piece: two steps of k = 2
      const float4 av = *reinterpret_cast<const float4*>(ar + ((c ^ sw) << 4));
      const float4 bv = *reinterpret_cast<const float4*>(br + ((c ^ sw) << 4));
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(hf ? av.y : av.x, hf ? bv.y : bv.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(hf ? av.w : av.z, hf ? bv.w : bv.z, acc, 0, 0, 0);
    }
  }
};

// e^x of a softmax cell in fp32 (hardware exponential of x log2 e): the logits come off the matrix cores with
// fp32 accumulation, so a cell carries a relative error of about 1e-6 already, and an fp64 exponential (some forty
// instructions) bought nothing. -inf gives 0.
__device__ __forceinline__ float exp2_f32(double x) { return __builtin_amdgcn_exp2f((float)(x * 1.4426950408889634)); }

// Leaves the head-summed map tile (rows I*64.., columns J*64..) in Ms[r * 65 + c] as doubles;
// cells above the diagonal or outside the chunk are 0. Called by all 256 threads; Ms doubles as
// the staging area of the operands (2 x 16 KB) before the tile values are written.
template <int DT, int KIND>
__device__ __forceinline__ void compute_tile(const SegArgs& a, int p, int I, int J, double* Ms) {
  typedef typename Elt<DT>::type T;
  const Dims& D = a.D;
  const int sl = p / D.Hkv, h = p - sl * D.Hkv, bi = a.batch_off + sl;
  const int seq = a.bp.seq[bi], c0 = a.bp.c0[bi];
  const int L = a.n_new, d = D.d;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wi = wave >> 1, wj = wave & 1, hf = lane >> 5, l32 = lane & 31;
  const int slot = slot_of(D, a.layer, seq, h);
  const T* Kc = reinterpret_cast<const T*>(a.k_arena) + arena_off(D, slot) + (size_t)chunk_tok_row(D, c0, c0) * d;
  const T* Qb = a.q_seg ? reinterpret_cast<const T*>(a.q_seg) + (size_t)bi * L * D.Hq * d + (size_t)h * D.G * d : nullptr;
  const int n_h = a.q_seg ? D.G : 1;
  const int nkc = d * (int)sizeof(T) / 256;                  // 256-byte pieces per row
  unsigned char* abuf = reinterpret_cast<unsigned char*>(Ms);
  unsigned char* bbuf = abuf + 16384;
  const double scale = 1.0 / sqrt((double)d);
  const int jcol = J * 64 + wj * 32 + l32;
  constexpr bool logit = KIND == LTRI_MAP_LOGIT;
  double m[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) m[v] = 0.0;
  f32x16_t acc = {0};
  for (int g = 0; g < n_h; ++g) {
    if constexpr (!logit) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    }
    for (int kc = 0; kc < nkc; ++kc) {
      if (Qb) stage_rows<T>(abuf, Qb + (size_t)g * d, (size_t)D.Hq * d, I * 64, L, kc);
      else    stage_rows<T>(abuf, Kc, (size_t)d, I * 64, L, kc);
      stage_rows<T>(bbuf, Kc, (size_t)d, J * 64, L, kc);
      __syncthreads();
      TileDot<DT>::run(abuf, bbuf, wi * 32, wj * 32, l32, hf, acc);
      __syncthreads();
    }
    if constexpr (!logit) {
      const double* lse = a.sc.lse + ((size_t)p * n_h + g) * a.Lp;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = I * 64 + wi * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
        m[v] += (double)exp2_f32((double)acc[v] * scale - lse[min(i, L - 1)]);
      }
    }
  }
  if constexpr (logit) {
#pragma unroll
    for (int v = 0; v < 16; ++v) m[v] = (double)acc[v] * scale;
  }
  if (I > J && (I + 1) * 64 <= L) {             // a whole tile below the diagonal: nothing to mask (uniform)
#pragma unroll
    for (int v = 0; v < 16; ++v) Ms[(wi * 32 + 8 * (v >> 2) + 4 * hf + (v & 3)) * 65 + wj * 32 + l32] = m[v];
    return;
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int rl = wi * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
    const int i = I * 64 + rl;
    const bool ok = (jcol <= i) && (i < L);
    Ms[rl * 65 + wj * 32 + l32] = ok ? m[v] : 0.0;
  }
}

// ---- theta as a percentile of the map (Sec. 4, "Hyperparameter Tuning") ----
// Exact selection of the cell of a given rank, without storing the map. The cells are ordered by an
// order-preserving 64-bit key. A pass over the recomputed tiles either counts the cells that share the key prefix
// found so far by their next 11-bit digit (LDS histogram, then integer atomics, so the result does not depend on
// the order of execution), after which a one-workgroup step picks the digit that holds the rank; or, once at
// most QUANT_LIST_CAP cells share the prefix, appends their keys to a list, and the one-workgroup step finishes
// the selection on the list. Three (tile pass, pick) pairs are launched, the first tile pass inside pass 1 of the
// segmentation (seg_tile_sums_kernel, whose sums do not depend on theta): for maps whose cells are not massively
// tied that is two counting passes and one collecting pass (one collecting pass for chunks of up to 180 tokens).
// A last kernel, one workgroup per problem, finishes whatever is left by walking the tiles itself (it returns at
// once when the selection is done): ties of more than QUANT_LIST_CAP cells within 2^-10 relative cost time there,
// not correctness.
// qstate[p] = {prefix, rank still to go, theta as double bits, status, -, -, -, -, lengths of the 16 sub-lists};
// status = cells that share the prefix | digits fixed << 32 | done << 63. The state is read and written at
// device scope: in the last kernel the same workgroup writes it and reads it back.
__device__ __forceinline__ uint64_t ascending_key(double v) {
  const uint64_t u = (uint64_t)__double_as_longlong(v + 0.0);        // -0.0 -> +0.0
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double key_to_double(uint64_t k) {
  const uint64_t u = (k >> 63) ? (k & 0x7fffffffffffffffull) : ~k;
  return __longlong_as_double((long long)u);
}
__host__ __device__ constexpr int quant_shift(int digit) { return 64 - QUANT_BITS * (digit + 1) > 0 ? 64 - QUANT_BITS * (digit + 1) : 0; }
__host__ __device__ constexpr int quant_width(int digit) { return 64 - QUANT_BITS * digit >= QUANT_BITS ? QUANT_BITS : 64 - QUANT_BITS * digit; }
constexpr int QUANT_PASSES = (64 + QUANT_BITS - 1) / QUANT_BITS;
constexpr int QUANT_TILE_PASSES = 3;                      // (tile pass, pick) pairs launched before the last kernel
constexpr unsigned long long QUANT_DONE = 1ull << 63;
__device__ __forceinline__ int quant_digits(unsigned long long status) { return (int)((status >> 32) & 0xFFull); }
__device__ __forceinline__ unsigned long long quant_count(unsigned long long status) { return status & 0xFFFFFFFFull; }
__device__ __forceinline__ unsigned long long qload(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void qstore(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct QuantShared {
  uint32_t hist[QUANT_BINS];
  unsigned long long part[256];
  unsigned long long prefix, rank, base, count;
  unsigned long long wtot[4];
  uint32_t len[QUANT_LISTS];
  uint32_t cnt;
  int digit;
};

__global__ __launch_bounds__(256) void quant_init_kernel(SegArgs a, unsigned long long rank, unsigned long long n_cells) {
  const int p = blockIdx.x;
  for (int b = threadIdx.x; b < QUANT_BINS; b += blockDim.x) a.sc.qhist[(size_t)p * QUANT_BINS + b] = 0u;
  if (threadIdx.x == 0) {
    unsigned long long* st = a.sc.qstate + (size_t)p * QUANT_STATE_WORDS;
    st[0] = 0ull;
    st[1] = rank;
    st[3] = n_cells;          // no digit fixed yet, not done
    for (int j = 0; j < QUANT_LISTS; ++j) st[8 + j] = 0ull;
  }
}

// One tile of a tile pass (all 256 threads), in two parts: quant_tile_clear before the tile is computed (a barrier
// lies between the two), quant_tile_cells once it is in Ms (which it only reads). status: the problem's status
// word as read by the caller.
__device__ __forceinline__ void quant_tile_clear(QuantShared& S) {
  for (int b = threadIdx.x; b < QUANT_BINS; b += blockDim.x) S.hist[b] = 0u;
  if (threadIdx.x == 0) S.cnt = 0u;
}
__device__ __forceinline__ void quant_tile_cells(const SegArgs& a, int p, int I, int J, unsigned long long status,
                                                 const double* Ms, QuantShared& S) {
  unsigned long long* st = a.sc.qstate + (size_t)p * QUANT_STATE_WORDS;
  const bool collect = quant_count(status) <= (unsigned long long)QUANT_LIST_CAP;
  const int digit = quant_digits(status);
  const int tid = threadIdx.x;
  const uint64_t prefix = qload(st + 0);
  const int hi = 64 - QUANT_BITS * digit;                 // bits from here up are the prefix (64: none yet)
  // a thread takes 16 consecutive cells of one row; a wavefront 64 consecutive rows (row pitch 65: no bank conflicts)
  const int r = tid & 63, c0 = (tid >> 6) * 16, y = I * 64 + r;
  auto matches = [&](int c, uint64_t& k) -> bool {
    const int x = J * 64 + c;
    if (!(x <= y && y < a.n_new)) return false;
    k = ascending_key(Ms[r * 65 + c]);
    return hi >= 64 || (k >> hi) == (prefix >> hi);
  };
  if (!collect) {
    // neighbouring cells often share the digit (the first digit is sign and exponent): runs are counted in a
    // register and added once
    const int shift = quant_shift(digit), width = quant_width(digit);
    uint32_t run_bin = 0xFFFFFFFFu, run = 0;
    for (int c = c0; c < c0 + 16; ++c) {
      uint64_t k;
      if (!matches(c, k)) continue;
      const uint32_t b = (uint32_t)(k >> shift) & ((1u << width) - 1u);
      if (b != run_bin) {
        if (run) atomicAdd(&S.hist[run_bin], run);
        run_bin = b; run = 0;
      }
      ++run;
    }
    if (run) atomicAdd(&S.hist[run_bin], run);
    __syncthreads();
    for (int b = tid; b < QUANT_BINS; b += blockDim.x)
      if (S.hist[b]) atomicAdd(&a.sc.qhist[(size_t)p * QUANT_BINS + b], S.hist[b]);
    return;
  }
  // the cells that share the prefix go to the list: count, reserve a run of the list, write
  uint32_t mine = 0;
  for (int c = c0; c < c0 + 16; ++c) { uint64_t k; mine += matches(c, k) ? 1u : 0u; }
  const uint32_t off = mine ? atomicAdd(&S.cnt, mine) : 0u;
  __syncthreads();
  const int sub = (I * (I + 1) / 2 + J) % QUANT_LISTS;   // the tile's sub-list
  if (tid == 0) S.base = S.cnt ? atomicAdd(&st[8 + sub], (unsigned long long)S.cnt) : 0ull;
  __syncthreads();
  unsigned long long at = S.base + off;
  unsigned long long* list = a.sc.qlist + ((size_t)p * QUANT_LISTS + sub) * QUANT_LIST_CAP;
  for (int c = c0; c < c0 + 16 && mine; ++c) {
    uint64_t k;
    if (matches(c, k)) { if (at < (unsigned long long)QUANT_LIST_CAP) list[at] = k; ++at; }
  }
}

template <int DT, int KIND>
__device__ __forceinline__ void quant_tile_step(const SegArgs& a, int p, int I, int J, unsigned long long status,
                                                double* Ms, QuantShared& S) {
  quant_tile_clear(S);
  compute_tile<DT, KIND>(a, p, I, J, Ms);
  __syncthreads();
  quant_tile_cells(a, p, I, J, status, Ms, S);
}

// The step after a tile pass (all 256 threads of one workgroup per problem): after a counting pass, the digit
// that holds the rank; after a collecting pass, the rest of the selection on the list (the same digit steps, over
// the list's keys instead of the tiles).
__device__ __forceinline__ void quant_pick_step(const SegArgs& a, int p, unsigned long long status, QuantShared& S) {
  const int tid = threadIdx.x;
  constexpr int PER = QUANT_BINS / 256;
  unsigned long long* st = a.sc.qstate + (size_t)p * QUANT_STATE_WORDS;
  const bool collected = quant_count(status) <= (unsigned long long)QUANT_LIST_CAP;
  uint32_t* gh = a.sc.qhist + (size_t)p * QUANT_BINS;
  // One digit step on the histogram in S.hist with S.part[t] = the sum of thread t's PER bins (all threads call
  // it after a barrier; S.prefix / S.rank hold the state and are updated, S.count gets the picked bin's count):
  // a scan of S.part over the workgroup finds the thread whose bins hold the rank, that thread walks its bins.
  auto pick_digit = [&](int digit) {
    const int lane = tid & 63, wave = tid >> 6;
    const unsigned long long own = S.part[tid], rank = S.rank;
    unsigned long long incl = own;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const unsigned long long v = __shfl_up(incl, o, 64);
      if (lane >= o) incl += v;
    }
    if (lane == 63) S.wtot[wave] = incl;
    __syncthreads();
    for (int w = 0; w < wave; ++w) incl += S.wtot[w];
    const unsigned long long excl = incl - own;
    // exactly one thread holds the rank; the last one also takes a rank beyond the total (cannot happen with
    // consistent counts)
    if (rank >= excl && (rank < incl || tid == 255)) {
      unsigned long long below = excl;
      int b = tid * PER;
      while (b < tid * PER + PER - 1 && below + S.hist[b] <= rank) { below += S.hist[b]; ++b; }
      S.prefix |= (uint64_t)b << quant_shift(digit);
      S.rank = rank - below;
      S.count = S.hist[b];
    }
    __syncthreads();
  };
  __syncthreads();
  if (tid == 0) { S.prefix = qload(st + 0); S.rank = qload(st + 1); S.digit = quant_digits(status); }
  if (!collected) {
    unsigned long long mine = 0;
    for (int e = 0; e < PER; ++e) {
      const uint32_t v = atomicExch(&gh[tid * PER + e], 0u);        // read and clear for the next pass
      S.hist[tid * PER + e] = v;
      mine += v;
    }
    S.part[tid] = mine;
    __syncthreads();
    const int digit = S.digit;
    pick_digit(digit);
    if (tid == 0) {
      qstore(st + 0, S.prefix);
      qstore(st + 1, S.rank);
      const bool last = digit + 1 == QUANT_PASSES;
      if (last) qstore(st + 2, (unsigned long long)__double_as_longlong(key_to_double(S.prefix)));
      qstore(st + 3, S.count | ((unsigned long long)(digit + 1) << 32) | (last ? QUANT_DONE : 0ull));
    }
    return;
  }
  // the lists hold every cell that shares the prefix: the remaining digits on the lists
  // (plain loads: nothing of the lists was in this compute unit's cache before they were written)
  const unsigned long long* lists = a.sc.qlist + (size_t)p * QUANT_LISTS * QUANT_LIST_CAP;
  if (tid < QUANT_LISTS) {
    const unsigned long long n_raw = qload(st + 8 + tid);
    S.len[tid] = (uint32_t)(n_raw < (unsigned long long)QUANT_LIST_CAP ? n_raw : (unsigned long long)QUANT_LIST_CAP);
  }
  __syncthreads();
  const int first_digit = S.digit;
  // the first 256 entries of every sub-list stay in registers over the digit steps (one independent load each);
  // longer sub-lists are walked again per digit
  unsigned long long kreg[QUANT_LISTS];
#pragma unroll
  for (int j = 0; j < QUANT_LISTS; ++j) kreg[j] = (uint32_t)tid < S.len[j] ? lists[(size_t)j * QUANT_LIST_CAP + tid] : 0ull;
  for (int digit = first_digit; digit < QUANT_PASSES; ++digit) {
    for (int e = 0; e < PER; ++e) S.hist[tid * PER + e] = 0u;
    __syncthreads();
    const unsigned long long prefix = S.prefix;
    const int shift = quant_shift(digit), width = quant_width(digit), hi = 64 - QUANT_BITS * digit;
    auto count_key = [&](unsigned long long k) {
      if (hi >= 64 || (k >> hi) == (prefix >> hi)) atomicAdd(&S.hist[(uint32_t)(k >> shift) & ((1u << width) - 1u)], 1u);
    };
#pragma unroll
    for (int j = 0; j < QUANT_LISTS; ++j)
      if ((uint32_t)tid < S.len[j]) count_key(kreg[j]);
    for (int j = 0; j < QUANT_LISTS; ++j) {
      const unsigned long long* list = lists + (size_t)j * QUANT_LIST_CAP;
      for (uint32_t i = tid + 256; i < S.len[j]; i += 256) count_key(list[i]);
    }
    __syncthreads();
    unsigned long long mine = 0;
    for (int e = 0; e < PER; ++e) mine += S.hist[tid * PER + e];
    S.part[tid] = mine;
    __syncthreads();
    pick_digit(digit);
  }
  if (tid == 0) {
    qstore(st + 0, S.prefix);
    qstore(st + 1, S.rank);
    qstore(st + 2, (unsigned long long)__double_as_longlong(key_to_double(S.prefix)));
    qstore(st + 3, QUANT_DONE);
  }
}

template <int DT, int KIND>
__global__ __launch_bounds__(256) void quant_tile_kernel(SegArgs a) {
  __shared__ double Ms[64 * 65];
  __shared__ QuantShared S;
  const int p = blockIdx.y;
  const unsigned long long status = qload(a.sc.qstate + (size_t)p * QUANT_STATE_WORDS + 3);
  if (status & QUANT_DONE) return;                        // the same for every workgroup of the problem
  int I, J;
  tile_decode(blockIdx.x, I, J);
  quant_tile_step<DT, KIND>(a, p, I, J, status, Ms, S);
}

__global__ __launch_bounds__(256) void quant_pick_kernel(SegArgs a) {
  __shared__ QuantShared S;
  const int p = blockIdx.x;
  const unsigned long long status = qload(a.sc.qstate + (size_t)p * QUANT_STATE_WORDS + 3);
  if (status & QUANT_DONE) return;
  quant_pick_step(a, p, status, S);
}

// Whatever the three launched pairs left undone, one workgroup per problem walking all tiles itself.
template <int DT, int KIND>
__global__ __launch_bounds__(256) void quant_finish_kernel(SegArgs a) {
  __shared__ double Ms[64 * 65];
  __shared__ QuantShared S;
  const int p = blockIdx.x;
  for (int it = 0; it < QUANT_PASSES; ++it) {
    const unsigned long long status = qload(a.sc.qstate + (size_t)p * QUANT_STATE_WORDS + 3);
    if (status & QUANT_DONE) return;                      // uniform: every thread reads the same word
    for (int t = 0; t < a.ntiles; ++t) {
      int I, J;
      tile_decode(t, I, J);
      quant_tile_step<DT, KIND>(a, p, I, J, status, Ms, S);
      __syncthreads();
    }
    quant_pick_step(a, p, status, S);
    __syncthreads();
  }
}

// ---- pass 1: per-tile row sums, suffix-scanned column sums, total ----
// QUANT (theta as a percentile of the map): the first tile pass of the selection rides here, on the same tile; the
// sums do not depend on theta.
template <int DT, int KIND, bool QUANT>
__global__ __launch_bounds__(256) void seg_tile_sums_kernel(SegArgs a) {
  __shared__ double Ms[64 * 65];
  __shared__ double cpart[4][64];
  __shared__ double rpart[4][64];
  __shared__ typename std::conditional<QUANT, QuantShared, int>::type S;
  const int p = blockIdx.y;
  int I, J;
  tile_decode(blockIdx.x, I, J);
  if constexpr (QUANT) quant_tile_clear(S);
  compute_tile<DT, KIND>(a, p, I, J, Ms);
  __syncthreads();
  if constexpr (QUANT) {
    const unsigned long long status = qload(a.sc.qstate + (size_t)p * QUANT_STATE_WORDS + 3);
    quant_tile_cells(a, p, I, J, status, Ms, S);       // (reads the tile; the sums below read it too)
  }
  const int tid = threadIdx.x;
  {                                       // row sums: four threads per row, 16 columns each; a wavefront takes
    const int r = tid & 63, qd = tid >> 6;  // 64 consecutive rows (row pitch 65: no bank conflicts)
    double s = 0.0;
#pragma unroll
    for (int c = 0; c < 16; ++c) s += Ms[r * 65 + qd * 16 + c];
    rpart[qd][r] = s;
  }
  {                                       // column sums: four threads per column, 16 rows each
    const int c = tid & 63, qd = tid >> 6;
    double s = 0.0;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += Ms[(qd * 16 + r) * 65 + c];
    cpart[qd][c] = s;
  }
  __syncthreads();
  if (tid >= 64 && tid < 128) {
    const int r = tid - 64;
    a.sc.rowsum[((size_t)p * a.nb + J) * a.Lp + I * 64 + r] = ((rpart[0][r] + rpart[1][r]) + rpart[2][r]) + rpart[3][r];
  }
  if (tid < 64) {                         // suffix scan over the 64 columns inside one wavefront
    double v = ((cpart[0][tid] + cpart[1][tid]) + cpart[2][tid]) + cpart[3][tid];
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double w = __shfl_down(v, o, 64);
      if (tid + o < 64) v += w;
    }
    // csuf is indexed [I][x]: block-row I's contribution restricted to this column block
    a.sc.csuf[((size_t)p * a.nb + I) * a.Lp + J * 64 + tid] = v;
    if (tid == 0) a.sc.tsum[((size_t)p * a.nb + I) * a.nb + J] = v;
  }
}

// ---- pass 2: the tile's carries from the sums of pass 1, then finish S inside the tile and reduce its
//      anti-diagonals ----
template <int DT, int KIND>
__global__ __launch_bounds__(256) void seg_tile_scan_kernel(SegArgs a) {
  __shared__ double Ms[64 * 65];
  __shared__ double qsum[4][64];       // sums of the four 16-wide pieces of a row / of a column
  __shared__ double cpart[4][64];      // the four threads' shares of a row's / a column's carry
  __shared__ double tpart[4];
  const int p = blockIdx.y;
  int I, J;
  tile_decode(blockIdx.x, I, J);
  const int tid = threadIdx.x, L = a.n_new;
  const bool whole = I > J && (I + 1) * 64 <= L;      // the tile lies below the diagonal and inside the chunk
  compute_tile<DT, KIND>(a, p, I, J, Ms);
  // The carries of this tile, from the sums of pass 1:
  //   row carry of row i        = sum of the tile row sums of row i over the tiles right of J (J < J' <= I),
  //   column carry of column x  = sum over the block rows above I (J <= I' < I) of their suffix-scanned column
  //                               sum at x, plus the totals of their tiles right of J (one number per tile).
  // Four threads share a row / a column, each every fourth term, with the same (row or column, quarter) a thread
  // has in the two scans below; the loads are requested here and used after the scans' first steps.
  const int li = tid & 63, part = tid >> 6;
  double rv[SEG_MAX_NB / 4], cv[SEG_MAX_NB / 4], tv[SEG_MAX_NB * SEG_MAX_NB / 256];
  {
    // every load is unconditional on a clamped (valid) index and masked afterwards: no branches, all in flight
    const double* rowsum = a.sc.rowsum + (size_t)p * a.nb * a.Lp + I * 64 + li;
    const double* csuf = a.sc.csuf + (size_t)p * a.nb * a.Lp + J * 64 + li;
    const double* tsum = a.sc.tsum + (size_t)p * a.nb * a.nb;
#pragma unroll
    for (int k = 0; k < SEG_MAX_NB / 4; ++k) {
      const int Jp = J + 1 + part + 4 * k, Ip = J + part + 4 * k;
      const double r = rowsum[min(Jp, I) * a.Lp], c = csuf[min(Ip, I) * a.Lp];
      rv[k] = Jp <= I ? r : 0.0;
      cv[k] = Ip < I ? c : 0.0;
    }
#pragma unroll
    for (int k = 0; k < SEG_MAX_NB * SEG_MAX_NB / 256; ++k) {      // tiles (I', J'') with J < J'' <= I' < I
      const int e = tid + 256 * k, Ip = e / SEG_MAX_NB, Jpp = e % SEG_MAX_NB;
      const double t = tsum[min(Ip, a.nb - 1) * a.nb + min(Jpp, a.nb - 1)];
      tv[k] = (Jpp > J && Jpp <= Ip && Ip < I) ? t : 0.0;
    }
  }
  __syncthreads();
  {                                     // rows: suffix sums towards the left, four threads per row; a wavefront
    const int r = li, qd = part;        // takes 64 consecutive rows (row pitch 65: no bank conflicts)
    double v[16];                       // the thread's cells stay in registers between the two steps
#pragma unroll
    for (int c = 0; c < 16; ++c) v[c] = Ms[r * 65 + qd * 16 + c];
    double s = 0.0;
#pragma unroll
    for (int c = 0; c < 16; ++c) s += v[c];
    double rs = 0.0;
#pragma unroll
    for (int k = 0; k < SEG_MAX_NB / 4; ++k) rs += rv[k];
    qsum[qd][r] = s;
    cpart[qd][r] = rs;
    __syncthreads();
    double run = ((cpart[0][r] + cpart[1][r]) + cpart[2][r]) + cpart[3][r];      // the row carry
    for (int q2 = 3; q2 > qd; --q2) run += qsum[q2][r];
#pragma unroll
    for (int c = 15; c >= 0; --c) { run += v[c]; Ms[r * 65 + qd * 16 + c] = run; }
  }
  __syncthreads();
  {                                     // columns: prefix sums downwards, four threads per column
    const int c = li, qd = part;
    double w[16];                       // kept in registers between the two steps
#pragma unroll
    for (int r = 0; r < 16; ++r) w[r] = Ms[(qd * 16 + r) * 65 + c];
    double s = 0.0;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += w[r];
    double cs = 0.0;
#pragma unroll
    for (int k = 0; k < SEG_MAX_NB / 4; ++k) cs += cv[k];
    const double ts = wave_sum_f64((tv[0] + tv[1]) + (tv[2] + tv[3]));
    qsum[qd][c] = s;
    cpart[qd][c] = cs;
    if (c == 0) tpart[qd] = ts;
    __syncthreads();
    const int x = J * 64 + c;
    const int n_h = a.q_seg ? a.D.G : 1;
    // Eq. 5's theta per head, times the heads summed; a percentile of the map is already per summed cell
    const double th = a.D.theta_quantile > 0.0 ? __longlong_as_double((long long)a.sc.qstate[(size_t)p * QUANT_STATE_WORDS + 2])
                                               : (double)a.D.theta * (double)n_h;
    double run = (((cpart[0][c] + cpart[1][c]) + cpart[2][c]) + cpart[3][c]) +
                 (((tpart[0] + tpart[1]) + tpart[2]) + tpart[3]);      // the column carry
    for (int q2 = 0; q2 < qd; ++q2) run += qsum[q2][c];
    // tri(n) = n (n + 1) / 2 of n = y - x + 1 by increments, tri(n + 1) = tri(n) + n + 1: small integers, exact
    // in fp64 (cells with n <= 0 lie above the diagonal and are masked)
    const int n0 = I * 64 + qd * 16 - x;                            // n - 1 of the thread's first row
    double nd = (double)n0, tri = (double)(n0 * (n0 + 1) / 2);      // |n0| <= 2048: the product fits 32 bits
    if (whole) {                                                    // (uniform) nothing to mask
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        run += w[r];
        nd += 1.0;
        tri += nd;
        Ms[(qd * 16 + r) * 65 + c] = run - th * tri;                // Eq. 5
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = qd * 16 + r, y = I * 64 + rl;
        run += w[r];
        nd += 1.0;
        tri += nd;
        const double sv = run - th * tri;                           // Eq. 5
        Ms[rl * 65 + c] = (x <= y && y < L) ? sv : -INFINITY;
      }
    }
  }
  __syncthreads();
  {
    // Anti-diagonals xl + yl = t and t + 64 of the tile hold t + 1 and 63 - t cells: together one cell per
    // column xl, in row (t - xl) mod 64 (no wrap: the first of the two). Four threads share such a pair, 16
    // columns each, so every thread reads exactly 16 cells, all requested at once; a wavefront takes 64
    // consecutive t (row pitch 65: no bank conflicts). Ties go to the larger x.
    const int t = li, q = part;
    double v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) { const int xl = 16 * q + j; v[j] = Ms[((t - xl) & 63) * 65 + xl]; }
    double bestA = -INFINITY, bestB = -INFINITY;
    int xA = -1, xB = -1;
    if (whole) {                                                    // (uniform) every cell is a cell of the map
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int xl = 16 * q + j;
        const bool first = xl <= t;
        const bool upA = first && v[j] >= bestA, upB = !first && v[j] >= bestB;
        bestA = upA ? v[j] : bestA; xA = upA ? xl : xA;
        bestB = upB ? v[j] : bestB; xB = upB ? xl : xB;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int xl = 16 * q + j;
        const bool first = xl <= t, live = v[j] > -INFINITY;
        const bool upA = first && live && v[j] >= bestA, upB = !first && live && v[j] >= bestB;
        bestA = upA ? v[j] : bestA; xA = upA ? xl : xA;
        bestB = upB ? v[j] : bestB; xB = upB ? xl : xB;
      }
    }
    double* hb = &Ms[0];                // the tile is consumed: [2][4][64] partial maxima, then their columns
    int* hx = reinterpret_cast<int*>(hb + 512);
    __syncthreads();
    hb[q * 64 + t] = bestA; hb[256 + q * 64 + t] = bestB;
    hx[q * 64 + t] = xA;    hx[256 + q * 64 + t] = xB;
    __syncthreads();
    if (tid < 128) {                    // anti-diagonal tid: its four quarters, larger columns last
      const int o = (tid >> 6) * 256 + (tid & 63);
      double best = hb[o];
      int bx = hx[o];
#pragma unroll
      for (int k = 1; k < 4; ++k) {
        const double ob = hb[o + 64 * k];
        const int ox = hx[o + 64 * k];
        if (ox >= 0 && (bx < 0 || ob >= best)) { best = ob; bx = ox; }
      }
      a.sc.pscore[((size_t)p * a.ntiles + blockIdx.x) * 128 + tid] = best;
      a.sc.px[((size_t)p * a.ntiles + blockIdx.x) * 128 + tid] = bx >= 0 ? J * 64 + bx : -1;
    }
  }
}

// ---- pass 3: candidates -> greedy NMS -> cuts -> span table ----

// Appends the spans cut at cutlist[0..n_cuts) (chunk-local, first 0, last L) to the slot's table.
__device__ void append_spans(const Dims& D, const DevState& st, int slot, int c0, int L,
                             const int* cutlist, int n_cuts) {
  int32_t* meta = st.meta + (size_t)slot * META_WORDS;
  const int base = meta[META_N_SPANS];
  const int n_sp = n_cuts - 1;
  const bool fits = base + n_sp <= D.max_spans;
  if (fits) {
    for (int k = threadIdx.x; k < n_sp; k += blockDim.x) {
      st.span_start[(size_t)slot * D.max_spans + base + k] = c0 + cutlist[k];
      st.span_len[(size_t)slot * D.max_spans + base + k] = cutlist[k + 1] - cutlist[k];
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (!fits) atomicCAS(&st.err[0], 0, LTRI_ECAPACITY);
    meta[META_N_SPANS] = fits ? base + n_sp : base;
    meta[META_CHUNK_FIRST] = base;
    meta[META_CHUNK_NSP] = fits ? n_sp : 0;
    meta[META_CHUNK_START] = c0;
    meta[META_CHUNK_LEN] = L;
    // META_SEL_CNT / META_LIST_LEN / the token list stay as they are: the attention of the previous
    // chunk may still be reading them on another stream; the host refuses to attend before the
    // next retrieve has rewritten them
  }
}

// Pass 3a: per anti-diagonal s = x + y, merge the tiles' partial results (ties: larger x =
// shorter span) and keep the span if S > 0 (appendix "NMS Input Filtration"). One thread per
// anti-diagonal, many workgroups per problem: the partial results are ~100 bytes per
// anti-diagonal and tile, far more than one CU reads quickly. Output: an order key (ascending
// key = descending score: positive doubles order like their bit patterns) and x << 16 | y.
__global__ __launch_bounds__(256) void seg_merge_kernel(SegArgs a) {
  const int p = blockIdx.y, nb = a.nb, L = a.n_new;
  const int n_diag = 2 * L - 1;
  const int s = blockIdx.x * 256 + threadIdx.x;
  if (s >= n_diag) return;
  const double* pscore = a.sc.pscore + (size_t)p * a.ntiles * 128;
  const int32_t* px = a.sc.px + (size_t)p * a.ntiles * 128;
  double best = -INFINITY;
  int bx = -1;
  const int b = s >> 6;
  for (int bb = b; bb >= b - 1 && bb >= 0; --bb) {
    const int sloc = s - 64 * bb;
    if (sloc > 126 || bb > 2 * (nb - 1)) continue;          // (no tile has I + J > 2 (nb - 1))
    // at most 16 tiles lie on one block anti-diagonal; all their entries are loaded before
    // the comparison chain so that the loads are in flight together
    const int J0 = max(0, bb - (nb - 1));
    double vs[SEG_MAX_NB / 2];
    int xs[SEG_MAX_NB / 2];
#pragma unroll
    for (int q = 0; q < SEG_MAX_NB / 2; ++q) {
      const int J = J0 + q;
      const bool ok = 2 * J <= bb;
      const int Jc = ok ? J : J0, I = bb - Jc;
      const size_t idx = (size_t)(I * (I + 1) / 2 + Jc) * 128 + sloc;
      vs[q] = pscore[idx];
      xs[q] = ok ? px[idx] : -1;
    }
#pragma unroll
    for (int q = 0; q < SEG_MAX_NB / 2; ++q) {
      const double v = vs[q];
      const int x = xs[q];
      if (x >= 0 && (v > best || (v == best && x > bx))) { best = v; bx = x; }
    }
  }
  const bool is_cand = bx >= 0 && best > 0.0;
  a.sc.ckey[(size_t)p * SEG_MAX_DIAG + s] = is_cand ? ~(uint64_t)__double_as_longlong(best) : ~0ull;
  a.sc.cxy[(size_t)p * SEG_MAX_DIAG + s] = is_cand ? (((uint32_t)bx << 16) | (uint32_t)(s - bx)) : 0xFFFFFFFFu;
}

// Pass 3b: greedy NMS (Sec. 3.2) over the candidates in the order (score descending, x ascending,
// y ascending), then the partition. Taking the candidates in sorted order and skipping the
// suppressed ones is the same as repeatedly taking the best candidate still alive, and the number
// of kept spans is small, so no sort is done: every thread holds four candidates in registers;
// one round = a workgroup-wide minimum of the order key over the live candidates, the winner is
// kept, every candidate it suppresses (and the winner itself) dies. One workgroup per problem.
__global__ __launch_bounds__(1024) void seg_select_kernel(SegArgs a) {
  __shared__ __attribute__((aligned(16))) uint32_t kept[SEG_MAX_DIAG + 1];
  if (blockIdx.y > 0) {
    // Not a selection: running sums of the chunk's query and key rows (bf16, head_dim 128), which step 2 reads once
    // the spans are known. They need nothing of the segmentation, and this launch leaves all but a few compute
    // units idle, so they ride along here (gridDim.y - 1 workgroups per problem, dispatched after the selections).
    static_assert(sizeof(kept) >= 16 * 16 * 8 * sizeof(double), "staging of the running sums");
    running_sums_block<LTRI_BF16, 16>(a.D, a.bp, a.layer, a.batch_off, a.rs, (int)blockIdx.y - 1, blockIdx.x,
                                      reinterpret_cast<double*>(kept));
    return;
  }
  __shared__ uint64_t s_w1[2][16];
  __shared__ uint32_t s_w2[2][16];
  __shared__ uint8_t flags[SEG_MAX_L + 64];
  __shared__ int cutlist[SEG_MAX_L + 1];
  __shared__ int s_wtot[16];
  const Dims& D = a.D;
  const int p = blockIdx.x, sl = p / D.Hkv, h = p - sl * D.Hkv, bi = a.batch_off + sl;
  const int seq = a.bp.seq[bi], c0 = a.bp.c0[bi];
  const int L = a.n_new, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n_diag = 2 * L - 1;
  uint64_t e1[4];
  uint32_t e2[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    // consecutive anti-diagonals per thread and wavefront: spans that are kept cover the chunk region by region,
    // so whole wavefronts run out of live candidates and skip most of a round
    const int sd = 4 * tid + r;
    e1[r] = sd < n_diag ? a.sc.ckey[(size_t)p * SEG_MAX_DIAG + sd] : ~0ull;
    e2[r] = sd < n_diag ? a.sc.cxy[(size_t)p * SEG_MAX_DIAG + sd] : 0xFFFFFFFFu;
  }
  const int max_keep = D.max_keep;
  const float phi = D.phi;
  int nkept = 0;
  for (int round = 0;; ++round) {
    // best live candidate of the thread, the wavefront, the workgroup
    uint64_t b1 = e1[0];
    uint32_t b2 = e2[0];
#pragma unroll
    for (int r = 1; r < 4; ++r)
      if (key_less(e1[r], e2[r], b1, b2)) { b1 = e1[r]; b2 = e2[r]; }
    auto step = [](auto mc, uint64_t& k1, uint32_t& k2) {
      constexpr int M = decltype(mc)::value;
      const uint32_t lo = lane_xor_c<M>((uint32_t)k1), hi = lane_xor_c<M>((uint32_t)(k1 >> 32));
      const uint32_t o2 = lane_xor_c<M>(k2);
      const uint64_t o1 = ((uint64_t)hi << 32) | lo;
      if (key_less(o1, o2, k1, k2)) { k1 = o1; k2 = o2; }
    };
    // The minimum over lanes goes by the keys' upper 32 bits first (one exchange and one minimum per step instead
    // of three exchanges and a 96-bit comparison); when exactly one lane holds that minimum its whole key is read
    // from that lane, otherwise (a tie in the upper bits: rare) the full keys are reduced.
    auto hi_min = [](auto steps, uint32_t m) {
      constexpr int S = decltype(steps)::value;
      m = min(m, lane_xor_c<1>(m));
      m = min(m, lane_xor_c<2>(m));
      m = min(m, lane_xor_c<4>(m));
      m = min(m, lane_xor_c<8>(m));
      if constexpr (S > 4) {
        m = min(m, lane_xor_c<16>(m));
        m = min(m, lane_xor_c<32>(m));
      }
      return m;
    };
    const bool wave_alive = __ballot(b1 != ~0ull) != 0ull;       // uniform over the wavefront
    if (wave_alive) {
      const uint32_t hi = (uint32_t)(b1 >> 32);
      const uint32_t m = hi_min(std::integral_constant<int, 6>{}, hi);
      const uint64_t tie = __ballot(hi == m);
      if (__popcll(tie) == 1) {
        const int src = __ffsll((long long)tie) - 1;
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b1, src);
        b2 = (uint32_t)__builtin_amdgcn_readlane((int)b2, src);
        b1 = ((uint64_t)m << 32) | lo;
      } else {
        step(std::integral_constant<int, 1>{}, b1, b2);
        step(std::integral_constant<int, 2>{}, b1, b2);
        step(std::integral_constant<int, 4>{}, b1, b2);
        step(std::integral_constant<int, 8>{}, b1, b2);
        step(std::integral_constant<int, 16>{}, b1, b2);
        step(std::integral_constant<int, 32>{}, b1, b2);
      }
    }
    const int buf = round & 1;                   // two buffers: one barrier per round
    if (lane == 0) { s_w1[buf][wave] = b1; s_w2[buf][wave] = b2; }
    __syncthreads();
    // the best of the 16 wavefronts: one entry per lane of every row of 16 lanes
    uint64_t w1 = s_w1[buf][lane & 15];
    uint32_t w2 = s_w2[buf][lane & 15];
    {
      const uint32_t hi = (uint32_t)(w1 >> 32);
      const uint32_t m = hi_min(std::integral_constant<int, 4>{}, hi);
      const uint64_t tie = __ballot(hi == m) & 0xFFFFull;         // the first row of 16 lanes
      if (__popcll(tie) == 1) {
        const int src = __ffsll((long long)tie) - 1;
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)w1, src);
        w2 = (uint32_t)__builtin_amdgcn_readlane((int)w2, src);
        w1 = ((uint64_t)m << 32) | lo;
      } else {
        step(std::integral_constant<int, 1>{}, w1, w2);
        step(std::integral_constant<int, 2>{}, w1, w2);
        step(std::integral_constant<int, 4>{}, w1, w2);
        step(std::integral_constant<int, 8>{}, w1, w2);
      }
    }
    if (w1 == ~0ull) break;                      // nothing alive (uniform)
    if (tid == 0) kept[nkept] = w2;
    ++nkept;
    if (max_keep > 0 && nkept >= max_keep) break;
    const int kx = (int)(w2 >> 16), ky = (int)(w2 & 0xFFFFu);
    if (!wave_alive) continue;                   // nothing left to suppress in this wavefront
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int x = (int)(e2[r] >> 16), y = (int)(e2[r] & 0xFFFFu);
      // suppressed iff inter > phi * union on inclusive token counts, compared in fp32 with one
      // multiply (the host-side definition does the same); branch-free: one select per candidate
      const int inter = min(y, ky) - max(x, kx) + 1;
      const int uni = (y - x + 1) + (ky - kx + 1) - inter;
      const bool kill = (e2[r] == w2) | ((inter > 0) & ((float)inter > __fmul_rn(phi, (float)uni)));
      e1[r] = kill ? ~0ull : e1[r];
    }
  }
  // cuts: 0, L, both ends of every kept interval, and (retrieval by memory units) every unit edge
  for (int i = tid; i <= L; i += blockDim.x)
    flags[i] = (i == 0 || i == L || (D.unit > 0 && (c0 + i) % D.unit == 0)) ? 1 : 0;
  __syncthreads();
  for (int q = tid; q < nkept; q += blockDim.x) {
    const uint32_t kk = kept[q];
    flags[kk >> 16] = 1;
    flags[(kk & 0xFFFFu) + 1] = 1;
  }
  __syncthreads();
  // enumerate the set flags in increasing order: each wave scans a contiguous segment
  const int seg = (L + 1 + 15) / 16, s0 = wave * seg, s1 = min(L + 1, s0 + seg);
  int cnt = 0;
  for (int i0 = s0; i0 < s1; i0 += 64) {
    const int i = i0 + lane;
    const bool f = i < s1 && flags[i];
    cnt += __popcll(__ballot(f));
  }
  if (lane == 0) s_wtot[wave] = cnt;
  __syncthreads();
  int off = 0, total = 0;
  for (int w = 0; w < 16; ++w) { if (w < wave) off += s_wtot[w]; total += s_wtot[w]; }
  for (int i0 = s0; i0 < s1; i0 += 64) {
    const int i = i0 + lane;
    const bool f = i < s1 && flags[i];
    const uint64_t m = __ballot(f);
    if (f) cutlist[off + __popcll(m & ((1ull << lane) - 1ull))] = i;
    off += __popcll(m);
  }
  __syncthreads();
  append_spans(D, a.st, slot_of(D, a.layer, seq, h), c0, L, cutlist, total);
}

// ============================================================================
// Dynamic span index vectors (Sec. 3.3.2). After the chunk's spans are in the table:
//   votes v_x (Eq. 6) = column sums of the chunk's head-summed softmax map,
//   r_a = area of a span's triangle over that area plus its neighbours' (same rows to the left,
//         same columns below, or both),
//   index tokens = the round(len / e^(lambda (1 - r_a))) tokens of the span with the most votes
//         (Eq. 7, clamped), stored vector = sum of their keys (Eq. 8 is bilinear).
// The map is recomputed tile by tile as in the segmentation passes; all sums are fp64 in a fixed
// order. The scratch arrays of the segmentation passes are free by then and are reused:
// rowsum[J][i] = tile row sums, rcar[J][i] = tile row sums over the columns of row i's own span,
// csuf[I][x] = tile column sums.
// ============================================================================

// ---- pass 0 (softmax map: SOFTMAX segmentation, dynamic index vectors): row log-sum-exp of the
//      chunk's causal scores from the same matrix-core tiles as the map ----
// Per tile and head: the row maximum and the sum of exponentials relative to it (lpart[.][J][i][2]);
// a second kernel merges the pieces of a row over its tiles.
template <int DT>
__global__ __launch_bounds__(256) void lse_tile_kernel(SegArgs a) {
  typedef typename Elt<DT>::type T;
  __shared__ double Ms[64 * 65];
  __shared__ double rmax[4][64], rsum[4][64];
  const Dims& D = a.D;
  const int p = blockIdx.y;
  int I, J;
  tile_decode(blockIdx.x, I, J);
  const int sl = p / D.Hkv, h = p - sl * D.Hkv, bi = a.batch_off + sl;
  const int seq = a.bp.seq[bi], c0 = a.bp.c0[bi];
  const int L = a.n_new, d = D.d;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1, hf = lane >> 5, l32 = lane & 31;
  const int slot = slot_of(D, a.layer, seq, h);
  const T* Kc = reinterpret_cast<const T*>(a.k_arena) + arena_off(D, slot) + (size_t)chunk_tok_row(D, c0, c0) * d;
  const T* Qb = a.q_seg ? reinterpret_cast<const T*>(a.q_seg) + (size_t)bi * L * D.Hq * d + (size_t)h * D.G * d : nullptr;
  const int n_h = a.q_seg ? D.G : 1;
  const int nkc = d * (int)sizeof(T) / 256;
  unsigned char* abuf = reinterpret_cast<unsigned char*>(Ms);
  unsigned char* bbuf = abuf + 16384;
  const double scale = 1.0 / sqrt((double)d);
  const int jcol = J * 64 + wj * 32 + l32;
  for (int g = 0; g < n_h; ++g) {
    f32x16_t acc = {0};
    for (int kc = 0; kc < nkc; ++kc) {
      if (Qb) stage_rows<T>(abuf, Qb + (size_t)g * d, (size_t)D.Hq * d, I * 64, L, kc);
      else    stage_rows<T>(abuf, Kc, (size_t)d, I * 64, L, kc);
      stage_rows<T>(bbuf, Kc, (size_t)d, J * 64, L, kc);
      __syncthreads();
      TileDot<DT>::run(abuf, bbuf, wi * 32, wj * 32, l32, hf, acc);
      __syncthreads();
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rl = wi * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
      const int i = I * 64 + rl;
      Ms[rl * 65 + wj * 32 + l32] = (jcol <= i && i < L) ? (double)acc[v] * scale : -INFINITY;
    }
    __syncthreads();
    {                                     // four threads per row, 16 columns each; a wavefront takes 64
      const int r = tid & 63, qd = tid >> 6;    // consecutive rows (row pitch 65: no bank conflicts)
      double z[16];
      double mx = -INFINITY;
#pragma unroll
      for (int c = 0; c < 16; ++c) { z[c] = Ms[r * 65 + qd * 16 + c]; mx = fmax(mx, z[c]); }
      rmax[qd][r] = mx;
      __syncthreads();
      mx = fmax(fmax(rmax[0][r], rmax[1][r]), fmax(rmax[2][r], rmax[3][r]));
      double sm = 0.0;
      if (mx > -INFINITY) {
#pragma unroll
        for (int c = 0; c < 16; ++c) sm += (double)exp2_f32(z[c] - mx);
      }
      rsum[qd][r] = sm;
      __syncthreads();
      if (qd == 0) {
        double* o = a.sc.lpart + ((((size_t)p * n_h + g) * a.nb + J) * a.Lp + I * 64 + r) * 2;
        o[0] = mx; o[1] = ((rsum[0][r] + rsum[1][r]) + rsum[2][r]) + rsum[3][r];
      }
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void lse_reduce_kernel(SegArgs a) {
  const int p = blockIdx.y, nb = a.nb, Lp = a.Lp;
  const int n_h = a.q_seg ? a.D.G : 1;
  const int id = blockIdx.x * blockDim.x + threadIdx.x;        // (g, i) flattened
  if (id >= n_h * Lp) return;
  const int g = id / Lp, i = id - g * Lp, B = i / 64;
  const double* pr = a.sc.lpart + (((size_t)p * n_h + g) * nb * Lp + i) * 2;
  double mx = -INFINITY;
#pragma unroll 8
  for (int J = 0; J <= B; ++J) mx = fmax(mx, pr[(size_t)J * Lp * 2]);
  double sm = 0.0;
#pragma unroll 8
  for (int J = 0; J <= B; ++J) {
    const double m = pr[(size_t)J * Lp * 2], s2 = pr[(size_t)J * Lp * 2 + 1];
    if (m > -INFINITY) sm += s2 * exp(m - mx);
  }
  a.sc.lse[((size_t)p * n_h + g) * Lp + i] = i < a.n_new ? mx + log(sm) : 0.0;
}

// span (within the chunk) of every token; clears the chunk's index-token mask
__global__ __launch_bounds__(256) void dyn_token_span_kernel(SegArgs a) {
  const Dims& D = a.D;
  const int p = blockIdx.y, sl = p / D.Hkv, h = p - sl * D.Hkv, bi = a.batch_off + sl;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int first = meta[META_CHUNK_FIRST], nsp = meta[META_CHUNK_NSP], c0 = meta[META_CHUNK_START];
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < IDX_MASK_WORDS) a.st.idx_mask[(size_t)slot * IDX_MASK_WORDS + i] = 0u;
  if (i >= a.Lp) return;
  const int32_t* sstart = a.st.span_start + (size_t)slot * D.max_spans + first;
  int lo = 0, hi = nsp - 1;                       // last span that starts at or before token i
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (sstart[mid] - c0 <= i) lo = mid; else hi = mid - 1;
  }
  a.sc.tokspan[(size_t)p * a.Lp + i] = (i < a.n_new && nsp > 0) ? lo : -1;
}

// per tile of the softmax map: row sums, row sums inside the row's own span, column sums
template <int DT>
__global__ __launch_bounds__(256) void dyn_tile_kernel(SegArgs a) {
  __shared__ double Ms[64 * 65];
  __shared__ double cpart[4][64], rpart[4][64], ipart[4][64];
  __shared__ int rspan[64], cspan[64];
  const int p = blockIdx.y;
  int I, J;
  tile_decode(blockIdx.x, I, J);
  compute_tile<DT, LTRI_MAP_SOFTMAX>(a, p, I, J, Ms);
  const int tid = threadIdx.x;
  if (tid < 64) rspan[tid] = a.sc.tokspan[(size_t)p * a.Lp + I * 64 + tid];
  else if (tid < 128) cspan[tid - 64] = a.sc.tokspan[(size_t)p * a.Lp + J * 64 + tid - 64];
  __syncthreads();
  {                                       // rows: four threads per row, 16 columns each; a wavefront takes 64
    const int r = tid & 63, qd = tid >> 6;  // consecutive rows (row pitch 65: no bank conflicts)
    const int mine = rspan[r];
    double s = 0.0, sin = 0.0;
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      const double v = Ms[r * 65 + qd * 16 + c];
      s += v;
      sin += cspan[qd * 16 + c] == mine ? v : 0.0;
    }
    rpart[qd][r] = s;
    ipart[qd][r] = sin;
  }
  {                                       // columns: four threads per column, 16 rows each
    const int c = tid & 63, qd = tid >> 6;
    double s = 0.0;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += Ms[(qd * 16 + r) * 65 + c];
    cpart[qd][c] = s;
  }
  __syncthreads();
  if (tid < 64) {
    a.sc.csuf[((size_t)p * a.nb + I) * a.Lp + J * 64 + tid] =
        ((cpart[0][tid] + cpart[1][tid]) + cpart[2][tid]) + cpart[3][tid];
  } else if (tid < 128) {
    const int r = tid - 64;
    a.sc.rowsum[((size_t)p * a.nb + J) * a.Lp + I * 64 + r] = ((rpart[0][r] + rpart[1][r]) + rpart[2][r]) + rpart[3][r];
    a.sc.rcar[((size_t)p * a.nb + J) * a.Lp + I * 64 + r] = ((ipart[0][r] + ipart[1][r]) + ipart[2][r]) + ipart[3][r];
  }
}

// per token: vote (column sum over the tiles below), row sum inside its span, whole row sum
__global__ __launch_bounds__(256) void dyn_reduce_kernel(SegArgs a) {
  const int p = blockIdx.y, nb = a.nb, Lp = a.Lp;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= Lp) return;
  const int B = i / 64;
  double v = 0.0, rin = 0.0, rall = 0.0;
#pragma unroll 8
  for (int I = B; I < nb; ++I) v += a.sc.csuf[((size_t)p * nb + I) * Lp + i];
#pragma unroll 8
  for (int J = 0; J <= B; ++J) {
    rin += a.sc.rcar[((size_t)p * nb + J) * Lp + i];
    rall += a.sc.rowsum[((size_t)p * nb + J) * Lp + i];
  }
  double* dyn = a.sc.dyn + (size_t)p * 3 * Lp;
  dyn[i] = v; dyn[Lp + i] = rin; dyn[2 * Lp + i] = rall;
}

// order key of a vote: smaller key = more votes
__device__ __forceinline__ uint64_t vote_key(double s) {
  const uint64_t u = (uint64_t)__double_as_longlong(s + 0.0);
  const uint64_t up = (u >> 63) ? ~u : (u | 0x8000000000000000ull);
  return ~up;
}

// per span: area ratio, number of index tokens (Eq. 7), the tokens, the sum of their keys
template <int DT>
__global__ __launch_bounds__(1024) void dyn_span_kernel(SegArgs a) {
  typedef typename Elt<DT>::type T;
  __shared__ double part[16][128];
  __shared__ uint64_t skey[SEG_MAX_L];
  __shared__ uint16_t spos[SEG_MAX_L];
  __shared__ uint32_t smask[IDX_MASK_WORDS + 1];
  __shared__ double red[3][16];
  __shared__ int s_count, s_mlo, s_mhi;
  __shared__ int s_cnt[SEG_MAX_L];                     // Eq. 7 counts of the spans of one memory block
  const Dims& D = a.D;
  const int p = blockIdx.y, sl = p / D.Hkv, h = p - sl * D.Hkv, bi = a.batch_off + sl;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int first = meta[META_CHUNK_FIRST], nsp = meta[META_CHUNK_NSP], c0 = meta[META_CHUNK_START];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double* dyn = a.sc.dyn + (size_t)p * 3 * a.Lp;
  const T* Kb = reinterpret_cast<const T*>(a.k_arena) + arena_off(D, slot);
  uint32_t* gmask = a.st.idx_mask + (size_t)slot * IDX_MASK_WORDS;
  for (int q = blockIdx.x; q < nsp; q += gridDim.x) {
    const int sid = first + q;
    const int start = a.st.span_start[(size_t)slot * D.max_spans + sid];
    const int len = a.st.span_len[(size_t)slot * D.max_spans + sid];
    const int a0 = start - c0;                          // chunk-local
    // sums over the span's tokens in a fixed order: per thread, per wave, then over the waves
    double sv = 0.0, sin = 0.0, sall = 0.0;
    for (int t = tid; t < len; t += blockDim.x) {
      sv += dyn[a0 + t]; sin += dyn[a.Lp + a0 + t]; sall += dyn[2 * a.Lp + a0 + t];
    }
    sv = wave_sum_f64(sv); sin = wave_sum_f64(sin); sall = wave_sum_f64(sall);
    if (lane == 0) { red[0][wave] = sv; red[1][wave] = sin; red[2][wave] = sall; }
    for (int w = tid; w < IDX_MASK_WORDS + 1; w += blockDim.x) smask[w] = 0u;
    __syncthreads();
    if (tid == 0) {
      double votes = 0.0, tri = 0.0, rows = 0.0;
      for (int w = 0; w < 16; ++w) { votes += red[0][w]; tri += red[1][w]; rows += red[2][w]; }
      // triangle + row neighbours = the span's rows; triangle + column neighbours = its votes
      const double den = D.ratio_mode == LTRI_RATIO_ROW ? rows
                       : D.ratio_mode == LTRI_RATIO_COL ? votes : rows + votes - tri;
      const double r_a = tri / den;
      const double r_v = 1.0 / exp(D.lambda * (1.0 - r_a));
      int n = (int)rint((double)len * r_v);
      n = max(n, D.index_min);
      if (D.index_max > 0) n = min(n, D.index_max);
      s_count = max(1, min(n, len));
    }
    if (D.index_block_max > 0) {
      // A budget of index vectors per memory block (the piece of a unit inside this chunk), shared over the
      // block's spans: every span of the block gets its own count by one and the same routine (one wavefront
      // per span, so that all workgroups of a block agree to the bit), then the largest counts are levelled
      // down to the highest level that fits and what is left goes to the earliest spans still short.
      __syncthreads();
      if (tid == 0) {
        const int blk = start / D.unit;
        int lo = q, hi = q;
        while (lo > 0 && a.st.span_start[(size_t)slot * D.max_spans + first + lo - 1] / D.unit == blk) --lo;
        while (hi + 1 < nsp && a.st.span_start[(size_t)slot * D.max_spans + first + hi + 1] / D.unit == blk) ++hi;
        s_mlo = lo; s_mhi = hi;
      }
      __syncthreads();
      const int mlo = s_mlo, mhi = s_mhi;
      for (int m = mlo + wave; m <= mhi; m += 16) {
        const int ms = a.st.span_start[(size_t)slot * D.max_spans + first + m] - c0;
        const int ml = a.st.span_len[(size_t)slot * D.max_spans + first + m];
        double v0 = 0.0, v1 = 0.0, v2 = 0.0;
        for (int t = lane; t < ml; t += 64) { v0 += dyn[ms + t]; v1 += dyn[a.Lp + ms + t]; v2 += dyn[2 * a.Lp + ms + t]; }
        v0 = wave_sum_f64(v0); v1 = wave_sum_f64(v1); v2 = wave_sum_f64(v2);
        if (lane == 0) {
          const double den = D.ratio_mode == LTRI_RATIO_ROW ? v2 : D.ratio_mode == LTRI_RATIO_COL ? v0 : v2 + v0 - v1;
          const double r_v = 1.0 / exp(D.lambda * (1.0 - v1 / den));
          int n = (int)rint((double)ml * r_v);
          n = max(n, D.index_min);
          if (D.index_max > 0) n = min(n, D.index_max);
          s_cnt[m - mlo] = max(1, min(n, ml));
        }
      }
      __syncthreads();
      if (tid == 0) {
        const int nm = mhi - mlo + 1, budget = D.index_block_max;
        long long total = 0;
        int cmax = 1;
        for (int m = 0; m < nm; ++m) { total += s_cnt[m]; cmax = max(cmax, s_cnt[m]); }
        int mine = s_cnt[q - mlo];
        if (total > budget) {
          int lvl_lo = 1, lvl_hi = cmax;                  // the largest level whose levelled total fits (1 if none does)
          while (lvl_lo < lvl_hi) {
            const int mid = (lvl_lo + lvl_hi + 1) >> 1;
            long long sum = 0;
            for (int m = 0; m < nm; ++m) sum += min(s_cnt[m], mid);
            if (sum <= budget) lvl_lo = mid; else lvl_hi = mid - 1;
          }
          const int level = lvl_lo;
          long long sum = 0;
          for (int m = 0; m < nm; ++m) sum += min(s_cnt[m], level);
          long long left = budget - sum;
          int share = min(mine, level);
          for (int m = 0; m < nm && left > 0; ++m) {
            if (s_cnt[m] > level) {
              if (m == q - mlo) ++share;
              --left;
            }
          }
          mine = share;
        }
        s_count = mine;
      }
    }
    // tokens by votes: bitonic network over (key, position), ascending
    int npow = 2;
    while (npow < len) npow <<= 1;
    for (int t = tid; t < npow; t += blockDim.x) {
      skey[t] = t < len ? vote_key(dyn[a0 + t]) : ~0ull;
      spos[t] = (uint16_t)t;
    }
    __syncthreads();
    for (int k = 2; k <= npow; k <<= 1) {
      for (int j = k >> 1; j > 0; j >>= 1) {
        for (int t = tid; t < npow / 2; t += blockDim.x) {
          const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;
          const uint64_t ka = skey[lo], kb = skey[hi];
          const uint16_t pa = spos[lo], pb = spos[hi];
          const bool a_after_b = (ka > kb) | ((ka == kb) & (pa > pb));
          if (a_after_b == ((lo & k) == 0)) {
            skey[lo] = kb; skey[hi] = ka;
            spos[lo] = pb; spos[hi] = pa;
          }
        }
        __syncthreads();
      }
    }
    const int count = s_count;
    for (int r = tid; r < count; r += blockDim.x) {
      const int t = spos[r];
      atomicOr(&smask[t >> 5], 1u << (t & 31));
    }
    __syncthreads();
    // the chunk's mask (spans share words at their edges)
    for (int w = tid; w <= (len - 1) >> 5; w += blockDim.x) {
      const uint32_t m = smask[w];
      if (m) {
        const int bit = a0 + 32 * w;                    // chunk-local bit of smask word w, bit 0
        const int sh = bit & 31;
        atomicOr(&gmask[bit >> 5], m << sh);
        if (sh && (bit >> 5) + 1 < IDX_MASK_WORDS) atomicOr(&gmask[(bit >> 5) + 1], m >> (32 - sh));
      }
    }
    T* rep = reinterpret_cast<T*>(a.st.krep) + ((size_t)slot * D.max_spans + sid) * D.d;
    span_mean_block<DT>(Kb + (size_t)chunk_tok_row(D, c0, start) * D.d, (size_t)D.d, 1, len, D.d, rep, part, nullptr, smask, 0);
  }
}

// ---- chunks of one token: a single span, its key is its own representative ----
struct SingleArgs { Dims D; DevState st; const void* k_arena; int layer; int seq_count; BatchPos bp; };

template <int DT>
__global__ __launch_bounds__(64) void append_single_kernel(SingleArgs a) {
  typedef typename Elt<DT>::type T;
  const Dims& D = a.D;
  const int p = blockIdx.x, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int seq = a.bp.seq[bi], c0 = a.bp.c0[bi];
  const int slot = slot_of(D, a.layer, seq, h);
  int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int base = meta[META_N_SPANS];
  const bool fits = base + 1 <= D.max_spans;
  if (fits) {
    const T* krow = reinterpret_cast<const T*>(a.k_arena) + arena_off(D, slot) + (size_t)chunk_tok_row(D, c0, c0) * D.d;
    T* rep = reinterpret_cast<T*>(a.st.krep) + ((size_t)slot * D.max_spans + base) * D.d;
    for (int c = threadIdx.x; c < D.d; c += 64) rep[c] = krow[c];
  }
  if (threadIdx.x == 0) {
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
}

// ---- caller-supplied boundaries ----
struct BoundsArgs { Dims D; DevState st; const int32_t* bounds; int layer, seq, c0, n_new; };

__global__ __launch_bounds__(256) void append_bounds_kernel(BoundsArgs a) {
  const Dims& D = a.D;
  const int h = blockIdx.x;
  const int32_t* cut = a.bounds + (size_t)h * (D.chunk_max + 1);
  const int n_cuts = a.bounds[(size_t)D.Hkv * (D.chunk_max + 1) + h];
  append_spans(D, a.st, slot_of(D, a.layer, a.seq, h), a.c0, a.n_new, cut, n_cuts);
}

// ---- representative keys: mean of the span's K rows, rounded once to the dtype ----
struct RepArgs { Dims D; DevState st; const void* k_arena; int layer; int seq_count; BatchPos bp; };

template <int DT>
__global__ __launch_bounds__(1024) void rep_keys_kernel(RepArgs a) {
  typedef typename Elt<DT>::type T;
  __shared__ double part[16][128];
  const Dims& D = a.D;
  const int p = blockIdx.y, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int first = meta[META_CHUNK_FIRST], nsp = meta[META_CHUNK_NSP], c0 = meta[META_CHUNK_START];
  const T* Kb = reinterpret_cast<const T*>(a.k_arena) + arena_off(D, slot);
  for (int q = blockIdx.x; q < nsp; q += gridDim.x) {
    const int sid = first + q;
    const int start = a.st.span_start[(size_t)slot * D.max_spans + sid];
    const int len = a.st.span_len[(size_t)slot * D.max_spans + sid];
    T* rep = reinterpret_cast<T*>(a.st.krep) + ((size_t)slot * D.max_spans + sid) * D.d;
    span_mean_block<DT>(Kb + (size_t)chunk_tok_row(D, c0, start) * D.d, (size_t)D.d, 1, len, D.d, rep, part);
  }
}

// ---- copies of a caller's chunk into the arenas ----
// Resident KV: the rows go to their tokens' places. Host-offloaded KV (Sec. 3.4 first step): the device keeps
// only the initial tokens and a ring of the latest tokens; every row is also written to the host arenas
// (device-visible pinned memory), from which step 3 fetches the rows it retrieves.
struct CopyArgs { Dims D; void* k_arena; void* v_arena; const void* k_chunk; const void* v_chunk;
                  int layer; int seq_count; int n_new; BatchPos bp; void* k_host; void* v_host; };

__global__ __launch_bounds__(256) void copy_chunk_kernel(CopyArgs a) {
  const Dims& D = a.D;
  const int p = blockIdx.y, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int c0 = a.bp.c0[bi];
  const size_t row_bytes = (size_t)D.d * D.elt;
  const int r16 = (int)(row_bytes / 16);                     // 16-byte pieces per row
  const size_t n16 = (size_t)a.n_new * r16;
  const size_t dst_off = (arena_off(D, slot) + (size_t)chunk_tok_row(D, c0, c0) * D.d) * D.elt;
  const size_t src_off = (size_t)p * a.n_new * row_bytes;
  const uint4* ks = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.k_chunk) + src_off);
  const uint4* vs = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.v_chunk) + src_off);
  uint4* kd = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.k_arena) + dst_off);
  uint4* vd = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.v_arena) + dst_off);
  if (!D.offload) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
      kd[i] = ks[i];
      vd[i] = vs[i];
    }
    return;
  }
  const size_t slot_bytes = arena_off(D, slot) * D.elt;
  uint4* kp = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.k_arena) + slot_bytes);     // row 0 of the slot's pool
  uint4* vp = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.v_arena) + slot_bytes);
  const size_t host_off = ((size_t)slot * (size_t)D.max_tokens + (size_t)c0) * row_bytes;
  uint4* kh = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.k_host) + host_off);
  uint4* vh = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.v_host) + host_off);
  const int ring = D.ring_mask + 1, pos0 = c0 & D.ring_mask;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
    const uint4 kv = ks[i], vv = vs[i];
    const int r = (int)(i / r16), piece = (int)(i - (size_t)r * r16);
    kd[i] = kv; vd[i] = vv;                                  // ring (running on into its mirror rows)
    if (pos0 + r >= ring) {                                  // the part past the ring's end, again at its start
      const size_t w = (size_t)(D.ring0 + pos0 + r - ring) * r16 + piece;
      kp[w] = kv; vp[w] = vv;
    }
    if (c0 + r < D.n_sink) {                                 // initial tokens keep rows of their own
      const size_t w = (size_t)(c0 + r) * r16 + piece;
      kp[w] = kv; vp[w] = vv;
    }
    kh[i] = kv; vh[i] = vv;                                  // host arenas: every token, in place
  }
}

// ---- host-offloaded KV: rows of the retrieved tokens, host arenas -> the staging rows of the device pool ----
// The context list is initial | retrieved | window; entry ns + j of the token list goes to pool row stage0 + j.
struct FetchArgs { Dims D; DevState st; void* k_pool; void* v_pool; const void* k_host; const void* v_host;
                   int layer; BatchPos bp; };

__global__ __launch_bounds__(256) void fetch_retrieved_kernel(FetchArgs a) {
  const Dims& D = a.D;
  const int p = blockIdx.y, bi = p / D.Hkv, h = p - bi * D.Hkv;
  const int slot = slot_of(D, a.layer, a.bp.seq[bi], h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int c0 = meta[META_CHUNK_START];
  const int ns = min(D.n_sink, c0), n_win = c0 - max(ns, c0 - D.window);
  const int n_ret = max(meta[META_LIST_LEN] - ns - n_win, 0);
  const int32_t* list = a.st.tok_list + (size_t)slot * D.list_cap + ns;
  const int r16 = D.d * D.elt / 16, rows_per_pass = 256 / r16;
  const int r_in = threadIdx.x / r16, piece = threadIdx.x - r_in * r16;
  const size_t row_bytes = (size_t)D.d * D.elt;
  const uint4* kh = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.k_host) + (size_t)slot * (size_t)D.max_tokens * row_bytes);
  const uint4* vh = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.v_host) + (size_t)slot * (size_t)D.max_tokens * row_bytes);
  uint4* kp = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.k_pool) + arena_off(D, slot) * D.elt) + (size_t)D.stage0 * r16;
  uint4* vp = reinterpret_cast<uint4*>(reinterpret_cast<char*>(a.v_pool) + arena_off(D, slot) * D.elt) + (size_t)D.stage0 * r16;
  for (int j = blockIdx.x * rows_per_pass + r_in; j < n_ret; j += gridDim.x * rows_per_pass) {
    const int tok = list[j];
    const uint4 kv = kh[(size_t)tok * r16 + piece];
    const uint4 vv = vh[(size_t)tok * r16 + piece];
    kp[(size_t)j * r16 + piece] = kv;
    vp[(size_t)j * r16 + piece] = vv;
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* p, size_t n16) {
  const uint4 z = {0, 0, 0, 0};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    p[i] = z;
}

// ============================================================================ launchers
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  const int blocks = (int)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
  fill_zero_kernel<<<blocks, 256, 0, s>>>(reinterpret_cast<uint4*>(p), n16);
  return hipGetLastError();
}

hipError_t launch_copy_chunk(const Dims& D, void* k_arena, void* v_arena, const void* k_chunk,
                             const void* v_chunk, int layer, const BatchPos& bp, int seq_count,
                             int n_new, void* k_host, void* v_host, hipStream_t s) {
  if (D.offload && (!k_host || !v_host)) return hipErrorInvalidValue;
  CopyArgs a{D, k_arena, v_arena, k_chunk, v_chunk, layer, seq_count, n_new, bp, k_host, v_host};
  const size_t n16 = (size_t)n_new * D.d * D.elt / 16;
  const int bx = (int)((n16 + 255) / 256 < 64 ? (n16 + 255) / 256 : 64);
  copy_chunk_kernel<<<dim3(bx > 0 ? bx : 1, seq_count * D.Hkv), 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_fetch_retrieved(const Dims& D, const DevState& st, void* k_pool, void* v_pool, const void* k_host,
                                  const void* v_host, int layer, const BatchPos& bp, int seq_count, hipStream_t s) {
  if (!D.offload || !k_host || !v_host) return hipErrorInvalidValue;
  FetchArgs a{D, st, k_pool, v_pool, k_host, v_host, layer, bp};
  // 16 workgroups per (sequence, KV head): 128 or more in all keep enough 16-byte reads in flight on the host link
  fetch_retrieved_kernel<<<dim3(16, seq_count * D.Hkv), 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_dynamic_reps(const Dims& D, const DevState& st, const DevScratch& sc, const void* k_arena,
                               const void* q_seg, int layer, const BatchPos& bp, int batch_off, int seq_count,
                               int n_new, bool lse_ready, hipEvent_t after_tiles, hipStream_t s) {
  SegArgs a;
  a.D = D; a.st = st; a.sc = sc; a.k_arena = k_arena; a.q_seg = q_seg; a.layer = layer;
  a.batch_off = batch_off; a.n_new = n_new;
  a.nb = (n_new + SEG_TB - 1) / SEG_TB; a.Lp = a.nb * SEG_TB; a.ntiles = a.nb * (a.nb + 1) / 2;
  a.bp = bp;
  a.sum_wgs = 0;
  a.rs = RunSums{};
  const int P = seq_count * D.Hkv;
  const bool bf = D.dtype == LTRI_BF16;
  dim3 gl((a.Lp + 255) / 256, P), gt(a.ntiles, P);
  if (!lse_ready) {
    const int n_h = q_seg ? D.G : 1;
    if (bf) lse_tile_kernel<LTRI_BF16><<<gt, 256, 0, s>>>(a);
    else    lse_tile_kernel<LTRI_F32><<<gt, 256, 0, s>>>(a);
    lse_reduce_kernel<<<dim3((n_h * a.Lp + 255) / 256, P), 256, 0, s>>>(a);
  }
  dyn_token_span_kernel<<<gl, 256, 0, s>>>(a);
  if (bf) dyn_tile_kernel<LTRI_BF16><<<gt, 256, 0, s>>>(a);
  else    dyn_tile_kernel<LTRI_F32><<<gt, 256, 0, s>>>(a);
  if (after_tiles) {                     // the last kernel that fills the chip is queued
    const hipError_t e = hipEventRecord(after_tiles, s);
    if (e != hipSuccess) return e;
  }
  dyn_reduce_kernel<<<gl, 256, 0, s>>>(a);
  dim3 gs(64, P);
  if (bf) dyn_span_kernel<LTRI_BF16><<<gs, 1024, 0, s>>>(a);
  else    dyn_span_kernel<LTRI_F32><<<gs, 1024, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_segment(const Dims& D, const DevState& st, const DevScratch& sc, const void* k_arena,
                          const void* q_seg, int layer, const BatchPos& bp, int batch_off, int seq_count,
                          int n_new, hipEvent_t after_tiles, const RunSums* sums, hipStream_t s) {
  SegArgs a;
  a.D = D; a.st = st; a.sc = sc; a.k_arena = k_arena; a.q_seg = q_seg; a.layer = layer;
  a.batch_off = batch_off; a.n_new = n_new;
  a.nb = (n_new + SEG_TB - 1) / SEG_TB; a.Lp = a.nb * SEG_TB; a.ntiles = a.nb * (a.nb + 1) / 2;
  a.bp = bp;
  a.sum_wgs = 0;
  a.rs = RunSums{};
  if (sums) {
    if (D.d != 128 || D.dtype != LTRI_BF16 || sums->n_q != n_new) return hipErrorInvalidValue;
    a.rs = *sums;
    a.sum_wgs = running_sums_blocks(a.rs, 16);
  }
  const int P = seq_count * D.Hkv;
  const bool bf = D.dtype == LTRI_BF16;
  dim3 gt(a.ntiles, P);
  if (D.seg_map == LTRI_MAP_SOFTMAX) {
    const int n_h = q_seg ? D.G : 1;
    if (bf) lse_tile_kernel<LTRI_BF16><<<gt, 256, 0, s>>>(a);
    else    lse_tile_kernel<LTRI_F32><<<gt, 256, 0, s>>>(a);
    lse_reduce_kernel<<<dim3((n_h * a.Lp + 255) / 256, P), 256, 0, s>>>(a);
  }
  // one instantiation per element type and map kind
  auto tiles = [&](auto dt, auto kind) {
    constexpr int DT = decltype(dt)::value, KIND = decltype(kind)::value;
    if (D.theta_quantile > 0.0) {
      const double n_cells = (double)n_new * (double)(n_new + 1) / 2.0;
      const unsigned long long rank = (unsigned long long)floor(D.theta_quantile * (n_cells - 1.0));
      quant_init_kernel<<<P, 256, 0, s>>>(a, rank, (unsigned long long)n_cells);
      seg_tile_sums_kernel<DT, KIND, true><<<gt, 256, 0, s>>>(a);      // pass 1 and the selection's first tile pass
      quant_pick_kernel<<<P, 256, 0, s>>>(a);
      for (int pass = 1; pass < QUANT_TILE_PASSES; ++pass) {
        quant_tile_kernel<DT, KIND><<<gt, 256, 0, s>>>(a);
        quant_pick_kernel<<<P, 256, 0, s>>>(a);
      }
      quant_finish_kernel<DT, KIND><<<P, 256, 0, s>>>(a);
    } else {
      seg_tile_sums_kernel<DT, KIND, false><<<gt, 256, 0, s>>>(a);
    }
    seg_tile_scan_kernel<DT, KIND><<<gt, 256, 0, s>>>(a);
  };
  using std::integral_constant;
  const bool lg = D.seg_map == LTRI_MAP_LOGIT;
  if (bf && lg)       tiles(integral_constant<int, LTRI_BF16>{}, integral_constant<int, LTRI_MAP_LOGIT>{});
  else if (bf)        tiles(integral_constant<int, LTRI_BF16>{}, integral_constant<int, LTRI_MAP_SOFTMAX>{});
  else if (lg)        tiles(integral_constant<int, LTRI_F32>{}, integral_constant<int, LTRI_MAP_LOGIT>{});
  else                tiles(integral_constant<int, LTRI_F32>{}, integral_constant<int, LTRI_MAP_SOFTMAX>{});
  // the kernels from here on use a few compute units each
  if (after_tiles) {
    const hipError_t e = hipEventRecord(after_tiles, s);
    if (e != hipSuccess) return e;
  }
  dim3 gm((2 * n_new - 1 + 255) / 256, P);
  seg_merge_kernel<<<gm, 256, 0, s>>>(a);
  seg_select_kernel<<<dim3(P, 1 + a.sum_wgs), 1024, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_append_single(const Dims& D, const DevState& st, const void* k_arena, int layer,
                                const BatchPos& bp, int seq_count, hipStream_t s) {
  SingleArgs a{D, st, k_arena, layer, seq_count, bp};
  if (D.dtype == LTRI_BF16) append_single_kernel<LTRI_BF16><<<seq_count * D.Hkv, 64, 0, s>>>(a);
  else                      append_single_kernel<LTRI_F32><<<seq_count * D.Hkv, 64, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_append_bounds(const Dims& D, const DevState& st, const DevScratch& sc, int layer,
                                int seq, int c0, int n_new, hipStream_t s) {
  BoundsArgs a{D, st, sc.bounds, layer, seq, c0, n_new};
  append_bounds_kernel<<<D.Hkv, 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_rep_keys(const Dims& D, const DevState& st, const void* k_arena, int layer,
                           const BatchPos& bp, int seq_count, int n_new, hipStream_t s) {
  RepArgs a{D, st, k_arena, layer, seq_count, bp};
  const int gx = n_new < 64 ? n_new : 64;
  dim3 g(gx, seq_count * D.Hkv);
  if (D.dtype == LTRI_BF16) rep_keys_kernel<LTRI_BF16><<<g, 1024, 0, s>>>(a);
  else                      rep_keys_kernel<LTRI_F32><<<g, 1024, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace ltri
