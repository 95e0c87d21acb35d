// Mean of a run of rows, used for the representative keys of new spans (Sec. 3.3.1, mean
// pooling) and for the query-span representatives of step 2. One workgroup of 16 wavefronts
// per span; every lane streams 16-byte pieces, so a long span has tens of KB in flight.
// Sums are fp64 in a fixed order (per lane, then across lanes, then across wavefronts): the
// result is deterministic, and exact before the final division for bf16 inputs.
#pragma once
#include "device_common.h"

namespace ltri {

// Accumulates rows r = 0 .. n_rows-1, row r = `inner` consecutive d-vectors of token r / inner:
// address base + (r / inner) * tok_stride + (r % inner) * d. Writes mean over tokens (sum over
// all rows divided by n_tokens) to out[0..d), or, when out_sum is given, the undivided fp64
// sums to out_sum[0..d). Called by all 1024 threads of a workgroup.
// With tokmask (global or LDS words, bit bit0 + t for token t) only the marked tokens are summed and
// the result is their sum, not a mean (the stored vector of a span's index tokens, Sec. 3.3.2).
template <int DT>
__device__ __forceinline__ void span_mean_block(const typename Elt<DT>::type* base, size_t tok_stride,
                                                int inner, int n_tokens, int d,
                                                typename Elt<DT>::type* out, double (*part)[128],
                                                double* out_sum = nullptr,
                                                const uint32_t* tokmask = nullptr, int bit0 = 0) {
  typedef typename Elt<DT>::type T;
  constexpr int EPP = 16 / (int)sizeof(T);           // elements per 16-byte piece
  const int R = d / EPP;                             // lanes per d-vector (16 or 32)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / R, piece = lane - sub * R;
  const int rpw = 64 / R;                            // rows per wavefront per load
  const int step = 16 * rpw;
  const int n_rows = n_tokens * inner;
  double acc[EPP];
#pragma unroll
  for (int e = 0; e < EPP; ++e) acc[e] = 0.0;
  for (int r0 = wave * rpw + sub; r0 < n_rows; r0 += 4 * step) {
    uint4 v[4];
    bool ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = r0 + u * step;
      ok[u] = r < n_rows;
      const int rr = ok[u] ? r : r0;
      const int tok = rr / inner, g = rr - tok * inner;
      if (tokmask) ok[u] = ok[u] && ((tokmask[(bit0 + tok) >> 5] >> ((bit0 + tok) & 31)) & 1u);
      v[u] = *reinterpret_cast<const uint4*>(base + (size_t)tok * tok_stride + (size_t)g * d + piece * EPP);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (ok[u]) {
        const T* pv = reinterpret_cast<const T*>(&v[u]);
#pragma unroll
        for (int e = 0; e < EPP; ++e) acc[e] += Elt<DT>::to_f64(pv[e]);
      }
    }
  }
  for (int o = R; o < 64; o <<= 1) {
#pragma unroll
    for (int e = 0; e < EPP; ++e) acc[e] += __shfl_xor(acc[e], o, 64);
  }
  if (lane < R) {
#pragma unroll
    for (int e = 0; e < EPP; ++e) part[wave][piece * EPP + e] = acc[e];
  }
  __syncthreads();
  if ((int)threadIdx.x < d) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < 16; ++w) s += part[w][threadIdx.x];
    // raw sum of a piece of a span, stored through to device scope: another workgroup of the same launch may
    // add the pieces up (the one that takes the last ticket)
    if (out_sum) __hip_atomic_store(out_sum + threadIdx.x, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else         out[threadIdx.x] = Elt<DT>::from_f64(tokmask ? s : s / (double)n_tokens);
  }
  __syncthreads();
}

}  // namespace ltri
