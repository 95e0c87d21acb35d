// Running sums of a chunk's query rows (summed over the query heads of a KV head) and key rows, for step 2 of long
// chunks with mean representatives: Q^R of a query span (Eq. 8's query side) and the mean key of a new span
// (Sec. 3.3.1) are each a difference of two running sums divided by the span's length, and running sums need no
// span boundaries, so they are taken while, or before, the chunk is segmented.
// Layout: out[problem][token][128] (fp64, `rows` rows per problem) holds, for token t, the sum of the rows of the
// tokens of t's block of RUNSUM_BLOCK tokens up to and including t; the reader adds the last rows of the earlier
// blocks. The key rows' sums follow `keys_off` elements behind the query rows'. head_dim 128 only. Sums of bf16
// values in fp64 are exact while the values of a column span less than 2^30 in magnitude over the chunk (8 bits
// each, 13 for the row count, 53 in all), so the result does not depend on the order of the additions and a
// difference of two running sums is the sum over the rows between them.
#pragma once
#include "device_common.h"

namespace ltri {

constexpr int RUNSUM_BLOCK = 128;

// Workgroups per problem that running_sums_block<DT, CG> is to be called by: one per block of query rows and
// column slab, one per two blocks of key rows (a key block is a quarter of the rows of a query block of the
// paper's model) and column slab.
__host__ __device__ inline int running_sums_blocks(const RunSums& r, int cg) {
  const int nblk = (r.n_q + RUNSUM_BLOCK - 1) / RUNSUM_BLOCK;
  return (nblk + (r.k_arena ? (nblk + 1) / 2 : 0)) * (16 / cg);
}

// One block of tokens (query or key rows) and CG of the 16 groups of 8 columns, for problem p = (sequence
// batch_off + p / Hkv, KV head p % Hkv). Called by all 64 * CG threads of a workgroup (CG = 4 or 16); wt: LDS,
// CG x CG x 8 doubles. A thread takes two tokens and 8 columns, the lanes of a wavefront CG column groups and
// 64 / CG pairs of tokens, so that every row is read in pieces of CG * 16 bytes.
template <int DT, int CG>
__device__ __forceinline__ void running_sums_one(const Dims& D, const BatchPos& bp, int layer, int batch_off,
                                                 const RunSums& r, int blk, int slab, bool keys, int p, double* wt) {
  typedef typename Elt<DT>::type T;
  constexpr int N = 16 / (int)sizeof(T);                // elements per 16-byte piece
  constexpr int NP = 8 / N;                             // pieces per 8 columns
  const int d = 128, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cgl = tid % CG, tp = tid / CG;              // column group inside the slab, pair of tokens
  const int col = (slab * CG + cgl) * 8;
  const int bi = batch_off + p / D.Hkv, h = p % D.Hkv;
  const int inner = keys ? 1 : D.G;                     // rows per token
  const size_t tok_stride = keys ? (size_t)d : (size_t)D.Hq * d;
  const T* base;
  if (keys) {
    const int c0 = bp.c0[bi];
    base = reinterpret_cast<const T*>(r.k_arena) + arena_off(D, slot_of(D, layer, bp.seq[bi], h)) +
           (size_t)chunk_tok_row(D, c0, c0) * d + col;
  } else {
    base = reinterpret_cast<const T*>(r.q) + (size_t)bi * r.n_q * D.Hq * d + (size_t)h * D.G * d + col;
  }
  double* out = r.out + (keys ? r.keys_off : (size_t)0) + (size_t)p * r.rows * d + col;
  const int t0 = blk * RUNSUM_BLOCK + 2 * tp;
  const bool ok0 = t0 < r.n_q, ok1 = t0 + 1 < r.n_q;
  const T* r0 = base + (size_t)min(t0, r.n_q - 1) * tok_stride;
  const T* r1 = base + (size_t)min(t0 + 1, r.n_q - 1) * tok_stride;
  double acc0[8], acc1[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc0[e] = acc1[e] = 0.0;
#pragma unroll 4
  for (int g = 0; g < inner; ++g) {
    uint4 v0[NP], v1[NP];
#pragma unroll
    for (int q = 0; q < NP; ++q) {
      v0[q] = reinterpret_cast<const uint4*>(r0 + (size_t)g * d)[q];
      v1[q] = reinterpret_cast<const uint4*>(r1 + (size_t)g * d)[q];
    }
    const T* e0 = reinterpret_cast<const T*>(v0);
    const T* e1 = reinterpret_cast<const T*>(v1);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      acc0[e] += Elt<DT>::to_f64(e0[e]);
      acc1[e] += Elt<DT>::to_f64(e1[e]);
    }
  }
  double ex[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    acc0[e] = ok0 ? acc0[e] : 0.0;
    acc1[e] = acc0[e] + (ok1 ? acc1[e] : 0.0);          // the pair's total
    // running sum over the wavefront's pairs of tokens (lanes CG apart)
    double v = acc1[e];
#pragma unroll
    for (int o = CG; o < 64; o <<= 1) {
      const double u = __shfl_up(v, o, 64);
      if (lane >= o) v += u;
    }
    const double u = __shfl_up(v, CG, 64);
    ex[e] = lane >= CG ? u : 0.0;
    if (lane >= 64 - CG) wt[(wave * CG + cgl) * 8 + e] = v;
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    double c0 = ex[e], c1 = ex[e + 1];
    for (int ww = 0; ww < wave; ++ww) {                 // CG wavefronts in all
      c0 += wt[(ww * CG + cgl) * 8 + e];
      c1 += wt[(ww * CG + cgl) * 8 + e + 1];
    }
    if (ok0) *reinterpret_cast<double2*>(out + (size_t)t0 * d + e) = make_double2(c0 + acc0[e], c1 + acc0[e + 1]);
    if (ok1) *reinterpret_cast<double2*>(out + (size_t)(t0 + 1) * d + e) = make_double2(c0 + acc1[e], c1 + acc1[e + 1]);
  }
}

// Workgroup `w` (0 .. running_sums_blocks - 1) of problem p.
template <int DT, int CG>
__device__ __forceinline__ void running_sums_block(const Dims& D, const BatchPos& bp, int layer, int batch_off,
                                                   const RunSums& r, int w, int p, double* wt) {
  constexpr int SLABS = 16 / CG;                        // workgroups that share a block's columns
  const int nblk = (r.n_q + RUNSUM_BLOCK - 1) / RUNSUM_BLOCK;
  const int slab = w % SLABS, wb = w / SLABS;
  if (wb < nblk) {
    running_sums_one<DT, CG>(D, bp, layer, batch_off, r, wb, slab, false, p, wt);
    return;
  }
  const int b0 = 2 * (wb - nblk);
  running_sums_one<DT, CG>(D, bp, layer, batch_off, r, b0, slab, true, p, wt);
  if (b0 + 1 < nblk) {                                  // uniform over the workgroup
    __syncthreads();                                    // wt is written again
    running_sums_one<DT, CG>(D, bp, layer, batch_off, r, b0 + 1, slab, true, p, wt);
  }
}

}  // namespace ltri
