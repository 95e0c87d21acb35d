// Step 3 on the device (Sec. 3.4 third step): exact attention of the query chunk over
// initial | retrieved | window tokens (read through the context token list built by step 2)
// and the chunk's own tokens (causal), plus the standalone gather of that context set.
//
// bf16 kernel: flash-style streaming over 64-key tiles on the matrix cores. A workgroup is
// eight wavefronts that share every K/V tile through LDS: the query heads of one KV head's
// group (GQA) times two 32-row sub-tiles, each wavefront with its 32 query rows in registers.
// Scores are computed transposed (S^T = K Q^T) so that one lane owns one query: the softmax
// statistics need a single cross-lane exchange and the probabilities are already laid out as
// the B operand of O^T = V^T P^T. The same kernel also attends over a part of the context
// only (the two parts of a step that overlaps steps 1 and 2), and splits the key range of
// a block of 2 to 4 query rows. One-token chunks (decode) have a kernel without LDS staging
// further down; fp32 contexts a plain one-wavefront-per-row kernel.
#include <hip/hip_ext.h>
#include "device_common.h"
#include <type_traits>

namespace ltri {

struct AttArgs {
  Dims D; DevState st; const void* k_arena; const void* v_arena; const void* q;
  void* out; float* lse; int layer; int seq_count; int n_q;
  int n_splits; float* part;             // short query blocks: the key range is split over workgroups
  int part_mode;                         // ATT_ALL, or one of the two parts of a two-part step
  const int32_t* loclist; int loc_cap;   // ATT_LOCAL: initial | window tokens per sequence [seq_count][loc_cap]
  const float* lse_a;                    // ATT_RETRIEVED: log-sum-exp of the first part, whose output is in `out`
  BatchPos bp;
};

// A step whose retrieved rows first have to come from host memory attends in two parts: the one that does
// not depend on the retrieval (initial and window tokens and the chunk itself) runs while the chunk is being
// segmented, its spans scored and the rows fetched; the retrieved tokens follow, and that launch folds the first part's result
// (already in `out`, with its log-sum-exp) into its own when it writes.
enum : int { ATT_ALL = 0, ATT_LOCAL = 1, ATT_RETRIEVED = 2 };

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// ---- bf16 kernel ----
// K and V tiles go from global memory straight into LDS (global_load_lds, 16 bytes per lane, no
// registers in between) through a ring of NS stages, so NS - 1 tiles are in flight while one is
// being consumed and a single barrier per tile suffices. Both tiles keep the row-major [key][d]
// layout of the arena; inside a 256-byte row the sixteen 16-byte pieces are permuted (XOR with a
// function of the row) so that the fragment reads are free of bank conflicts; the permutation is
// applied by choosing which piece each lane fetches. V^T fragments (A operand of
// O^T = V^T P^T) are read with the transposing LDS load: lane j of a 16-lane group passes the
// address of 4 consecutive d-columns of key row0 + j / 4, lane i receives column i of keys
// row0 .. row0 + 3.
// The DMA is issued through inline assembly because the compiler would otherwise wait for ALL
// outstanding DMA before any LDS read; completion is awaited by hand with s_waitcnt vmcnt(n),
// n = DMA loads requested later than the tile about to be used. Every wavefront issues the same
// number of requests in every iteration (its rows of one K/V tile and the token ids of its rows
// of a later tile; past the last tile the requests fetch the chunk's last row into a free stage),
// so n is one constant.
// The K fragments of a tile are requested together by hand (the compiler would serialise them
// once registers are tight) and consumed in four groups; the DMA requests of a later tile are
// issued between the groups, under the matrix products. The rescale of O is skipped while no
// lane's running maximum moves.
// The tile loop is cut into segments (context tiles, the ragged last context tile, chunk tiles
// below the diagonal, chunk tiles on the diagonal, tiles this wavefront cannot see) so that the
// body of each segment is straight-line code, with the masks compiled in or out.
typedef short s16x4_t __attribute__((ext_vector_type(4)));

constexpr int ATT_NW = 8;                       // wavefronts per workgroup of the bf16 kernel
constexpr int DMA_STAGE_BYTES = 32768;          // K tile 16 KB + V tile 16 KB
constexpr int TOK_SLOTS = 8;                    // ring of token-id tiles (> tokens-ahead distance)
constexpr int att_lds_bytes(int ns, int nw) { return ns * DMA_STAGE_BYTES + TOK_SLOTS * nw * 32; }

// 16 bytes per lane from base + off into LDS at lds_wave_base + 16 * lane. The idle cycle between the write of
// M0 and the load that uses it is the wait state the instruction set asks for; inside an assembly block the
// compiler does not add it.
__device__ __forceinline__ void dma16(const void* base, uint32_t off, uint32_t lds_wave_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_wave_base), "v"(off), "s"(base) : "m0");
}
// 4 bytes per lane
__device__ __forceinline__ void dma4(const void* base, uint32_t off, uint32_t lds_wave_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_wave_base), "v"(off), "s"(base) : "m0");
}

enum : int { MASK_NONE = 0, MASK_LIST_END = 1, MASK_CAUSAL = 2 };

// max of three. This file is compiled with -fno-honor-nans (scores are never NaN here), so fmaxf() carries no
// NaN-quieting copies and the compiler folds the pair into one v_max3_f32; being the compiler's own
// instruction, it gets the wait states it needs after matrix-core results and before lane permutes.
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// acc + lo + hi of a packed bf16 pair (one v_dot2c_f32_bf16)
__device__ __forceinline__ float pair_sum(uint32_t packed, float acc) {
  const bf16x2_t one = {(__bf16)1.0f, (__bf16)1.0f};
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, packed), one, acc, false);
}

// max over lanes l and l ^ 32 without an LDS round trip: the swap leaves the low half of v in
// both halves of r[0] and the high half in both halves of r[1]
__device__ __forceinline__ float pair_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// 16-byte LDS read issued by hand; LDS reads return in order, and the loop holds no scalar loads
// that could disturb the count awaited below
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <int OFF>
__device__ __forceinline__ u32x4_t lds_read16(uint32_t addr) {
  u32x4_t r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
// at most N LDS reads still outstanding; ties the four fragments about to be used to the wait
template <int N>
__device__ __forceinline__ void lds_wait(u32x4_t& a, u32x4_t& b, u32x4_t& c, u32x4_t& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}

// NW wavefronts per workgroup, each with 32 query rows of one head; NS ring stages.
template <int NW, int NS>
__global__ __launch_bounds__(64 * NW) void attend_bf16_kernel(AttArgs a) {
  constexpr int TOK_AHEAD = 2 * (NS - 1) + 1;       // token ids of tile t + TOK_AHEAD are requested in iteration t
  constexpr int NI = 16 / NW;                       // DMA row groups per wave and tile
  constexpr int LPT = 2 * NI;                       // K/V requests per lane and tile
  constexpr int IN_FLIGHT = (NS - 2) * (LPT + 1);   // requests that may be pending when a tile is used
  static_assert(NS >= 3 && NS <= 4 && TOK_AHEAD < TOK_SLOTS && NI == 2, "request pattern");
  extern __shared__ __attribute__((aligned(16))) unsigned char ring[];
  const Dims& D = a.D;
  const int HG = D.G < 4 ? D.G : 4;                 // heads of the group handled by this block
  const int RS = NW / HG;                           // row sub-tiles per block
  const int RPB = 32 * RS;                          // query rows per block
  const int gpk = D.G / HG;                         // blocks per KV head
  // KV head along x: consecutive workgroup ids go to different XCDs, so all query tiles of one
  // KV head run on one XCD and share its K/V rows in that XCD's L2
  const int bi = blockIdx.z, h = blockIdx.x / gpk, gsub = blockIdx.x - h * gpk;
  const int seq = a.bp.seq[bi], c0 = a.bp.c0[bi];
  const int L = a.n_q, d = 128;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int head = h * D.G + gsub * HG + (wave % HG);
  const int split = a.n_splits > 1 ? blockIdx.y : 0;
  // Query rows of the workgroup. The chunk's rows are cut into sub-tiles of 32; workgroup y takes RS / 2 of them
  // from the low end and RS / 2 from the high end (sub-tiles y RS / 2 .. and their mirror images), so that under
  // the causal mask every workgroup has about the same number of (sub-tile, chunk tile) pairs to compute: the
  // low sub-tiles stop early at their diagonal, the high ones walk on alone. With one sub-tile per workgroup
  // (RS == 1) rows are taken in order.
  const int nsub = (RPB == 32) ? (L + 31) / 32 : ((L + RPB - 1) / RPB) * RS;    // sub-tiles, padded to whole workgroups
  const int yb = a.n_splits > 1 ? 0 : (int)blockIdx.y;
  const int rs = wave / HG;
  const int sub = (RS == 1) ? yb : (rs < RS / 2 ? yb * (RS / 2) + rs : nsub - (yb + 1) * (RS / 2) + (rs - RS / 2));
  const int r0 = sub * 32;                          // first row of this wave
  const int rb_end = (RS == 1) ? min(L, r0 + 32) : min(L, (nsub - yb * (RS / 2)) * 32);   // past the last row of the workgroup
  const int slot = slot_of(D, a.layer, seq, h);
  const unsigned char* Kb = reinterpret_cast<const unsigned char*>(a.k_arena) + arena_off(D, slot) * 2;
  const unsigned char* Vb = reinterpret_cast<const unsigned char*>(a.v_arena) + arena_off(D, slot) * 2;
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  // the context list is initial | retrieved | window; the two parts of a two-part step read
  // initial | window from a list of their own, or the retrieved slice of the full list
  const int n_init = min(D.n_sink, c0), n_win = c0 - max(n_init, c0 - D.window);
  int list_len = meta[META_LIST_LEN];
  const int32_t* list = a.st.row_list + (size_t)slot * D.list_cap;
  if (a.part_mode == ATT_LOCAL) {
    list_len = n_init + n_win;
    list = a.loclist + (size_t)bi * a.loc_cap;
  } else if (a.part_mode == ATT_RETRIEVED) {
    list_len = max(list_len - n_init - n_win, 0);
    list += n_init;
  }
  const int n_ctx_tiles = (list_len + 63) / 64;
  const int crow0 = chunk_tok_row(D, c0, c0);       // row of the chunk's first token (the chunk's rows are consecutive)
  const int n_chunk_tiles = a.part_mode == ATT_RETRIEVED ? 0 : (rb_end + 63) / 64;
  const int n_tiles = n_ctx_tiles + n_chunk_tiles;
  // with splits, this workgroup takes the context tiles [tile0, tile1); the last split also takes the chunk's tiles
  const int tile0 = a.n_splits > 1 ? (int)((long long)split * n_ctx_tiles / a.n_splits) : 0;
  const int tile1 = (a.n_splits > 1 && split + 1 < a.n_splits) ? (int)((long long)(split + 1) * n_ctx_tiles / a.n_splits) : n_tiles;
  const uint32_t ring0 = (uint32_t)(uintptr_t)ring;
  const uint32_t tok0 = ring0 + NS * DMA_STAGE_BYTES + (uint32_t)wave * 32;       // this wave's 8 ids of slot 0
  const int32_t* tokring = reinterpret_cast<const int32_t*>(ring + NS * DMA_STAGE_BYTES) + wave * 8;

  // ---- requests ----
  // A wavefront fetches rows 4 NW i + 4 wave + lq (i < NI, lq = lane / 16) of every tile, lane
  // piece lp = lane % 16 of the row. The token ids of its own eight rows travel through LDS the
  // same way (lanes 0 .. 7, id j = 4 i + lq), TOK_AHEAD tiles ahead; no other wave reads them, so
  // the wave's own wait makes them visible. Tiles past the list read a dummy entry.
  auto request_tokens = [&](int u) {
    if (lane < 8) {
      const int row = 4 * NW * (lane >> 2) + 4 * wave + (lane & 3);
      dma4(list, (uint32_t)((u < n_ctx_tiles ? u * 64 : 0) + row) * 4u, tok0 + (uint32_t)(u % TOK_SLOTS) * (NW * 32));
    }
  };
  const int lq = lane >> 4, lp = lane & 15;
  uint32_t kpiece[NI], vpiece[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int row = 4 * NW * i + 4 * wave + lq;
    kpiece[i] = (uint32_t)((lp ^ (row & 15)) << 4);
    // V: LDS piece p' of a row holds global piece swap13(p' ^ ((row & 3) << 1)), swap13 = exchange of bits 1 and 3
    const int vp = lp ^ ((row & 3) << 1);
    vpiece[i] = (uint32_t)(((vp & 5) | ((vp & 2) << 2) | ((vp & 8) >> 2)) << 4);
  }
  // tokens of the rows this lane fetches in tile t (list padding is token 0, masked by position;
  // past the last tile: the chunk's last token)
  auto tile_tokens = [&](int t, int (&tok)[NI]) {
    if (t < n_ctx_tiles) {
#pragma unroll
      for (int i = 0; i < NI; ++i) tok[i] = tokring[(t % TOK_SLOTS) * (NW * 8) + 4 * i + lq];
    } else {
#pragma unroll
      for (int i = 0; i < NI; ++i) tok[i] = crow0 + min((t - n_ctx_tiles) * 64 + 4 * NW * i + 4 * wave + lq, L - 1);
    }
  };
  auto request_rows = [&](int t, int i, int tok) {
    const uint32_t dst = ring0 + (uint32_t)(t % NS) * DMA_STAGE_BYTES + (uint32_t)(4 * NW * i + 4 * wave) * 256;
    dma16(Kb, ((uint32_t)tok << 8) + kpiece[i], dst);
    dma16(Vb, ((uint32_t)tok << 8) + vpiece[i], dst + 16384u);
  };

  // ---- query fragments: B operand of S^T = K Q^T; lane (l32, hf) holds Q[row l32][16 kk + 8 hf ..] ----
  uint4 qf[8];
  {
    const uint16_t* Qb = reinterpret_cast<const uint16_t*>(a.q) + (size_t)bi * L * D.Hq * d;
    const int row = min(r0 + l32, L - 1);
    const uint16_t* qrow = Qb + ((size_t)row * D.Hq + head) * d;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = *reinterpret_cast<const uint4*>(qrow + kk * 16 + hf * 8);
  }
  // The fragments are "used" here so that the compiler's wait for these loads sits before the
  // loop: a wait for them inside the loop would also wait for every DMA request in flight.
#pragma unroll
  for (int kk = 0; kk < 8; ++kk)
    asm volatile("" ::"v"(qf[kk].x), "v"(qf[kk].y), "v"(qf[kk].z), "v"(qf[kk].w));

  f32x16_t o[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[mb][v] = 0.f;
  float m_run = -1e30f, l_run = 0.f;                // running maximum (log2 domain) and sum
  const float sc = 1.4426950408889634f / sqrtf((float)d);     // log2(e) / sqrt(d)

  // per-lane parts of the fragment addresses
  // K: row l32 (+ 32 kb), piece (2 kk + hf) ^ (row & 15) = ((2 kk) ^ (row & 14)) | (hf ^ (row & 1))
  const uint32_t kbase = (uint32_t)(l32 * 256 + ((hf ^ (l32 & 1)) << 4));
  const uint32_t kswz = (uint32_t)((l32 & 14) << 4);
  uint32_t koff[8];                                 // fragment kk of rows l32 and l32 + 32 (+ 8192)
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) koff[kk] = ring0 + kbase + (kswz ^ (uint32_t)(kk << 5));
  const int vj = lane & 15, vgq = (lane >> 4) & 1;
  const int vrow_in = 4 * hf + (vj >> 2);           // key row inside a group of 8
  // V: the fragment of d-block mb needs global piece 4 mb + 2 gq + x (x = (j & 3) / 2). In LDS it sits at
  // piece swap13(.) ^ swizzle = (gq << 3 | x) | ((mb & 1) << 2 | (mb >> 1) << 1) ^ swizzle: the two
  // 16-lane groups of a half-wave read different 128-byte halves of their rows (no bank conflicts
  // between them), and the four key rows of a group are spread by the swizzle in bits 1..2.
  const uint32_t vbase = (uint32_t)(vrow_in * 256 + (((vgq << 3) | ((vj & 3) >> 1)) << 4) + (vj & 1) * 8);
  const uint32_t vswz = (uint32_t)(((vrow_in & 3) << 1) << 4);
  uint32_t voff[4];                                 // d-block mb
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
    voff[mb] = ring0 + 16384u + vbase + (vswz ^ (uint32_t)((((mb & 1) << 2) | ((mb >> 1) << 1)) << 4));

  int tokreg[NI];                                   // tokens of the rows of the next tile to request

  // ---- one iteration: wait for tile t, barrier, S^T = K Q^T with the requests of tile t + NS - 1
  //      between the products, masks, online softmax (one query per lane pair), O^T += V^T P^T.
  //      compute = false: a tile this wavefront cannot see (requests, wait and barrier only) ----
  auto tile = [&](int t, auto mask_kind, auto compute_kind) {
    constexpr int MK = decltype(mask_kind)::value;
    constexpr bool COMPUTE = decltype(compute_kind)::value;
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(IN_FLIGHT) : "memory");
    __syncthreads();            // tile t is in LDS for every wave; tile t - 1's stage is free
    const uint32_t sbase = (uint32_t)(t % NS) * DMA_STAGE_BYTES;
    int toknext[NI];
    tile_tokens(t + NS, toknext);
    f32x16_t s[2];
    if constexpr (COMPUTE) {
      // all sixteen K fragments are requested at once (index 2 kk + kb) and used in groups of four
      u32x4_t kf[16];
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        kf[2 * kk] = lds_read16<0>(sbase + koff[kk]);
        kf[2 * kk + 1] = lds_read16<8192>(sbase + koff[kk]);
      }
      __builtin_amdgcn_s_setprio(2);               // matrix-core phases go first when both waves of a SIMD are ready
      const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      auto group = [&](int g) {
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
            s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[4 * g + 2 * k2 + kb]),
                                                            __builtin_bit_cast(bf16x8_t, qf[2 * g + k2]),
                                                            (g == 0 && k2 == 0) ? zero : s[kb], 0, 0, 0);
      };
      // the scheduling barriers keep each group's products between its wait and the next one
      lds_wait<12>(kf[0], kf[1], kf[2], kf[3]);     group(0); __builtin_amdgcn_sched_barrier(0);
      request_tokens(t + TOK_AHEAD);
      request_rows(t + NS - 1, 0, tokreg[0]);
      lds_wait<8>(kf[4], kf[5], kf[6], kf[7]);      group(1); __builtin_amdgcn_sched_barrier(0);
      request_rows(t + NS - 1, 1, tokreg[1]);
      lds_wait<4>(kf[8], kf[9], kf[10], kf[11]);    group(2); __builtin_amdgcn_sched_barrier(0);
      lds_wait<0>(kf[12], kf[13], kf[14], kf[15]);  group(3);
      __builtin_amdgcn_s_setprio(0);
    } else {
      request_tokens(t + TOK_AHEAD);
      request_rows(t + NS - 1, 0, tokreg[0]);
      request_rows(t + NS - 1, 1, tokreg[1]);
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) tokreg[i] = toknext[i];
    if constexpr (!COMPUTE) return;
    if constexpr (MK == MASK_CAUSAL) {
      const int k0 = (t - n_ctx_tiles) * 64;
      const int qi = r0 + l32;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int kp = k0 + kb * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
          if (kp > qi) s[kb][v] = -INFINITY;
        }
    } else if constexpr (MK == MASK_LIST_END) {
      const int nvalid = list_len - t * 64;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int kr = kb * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
          if (kr >= nvalid) s[kb][v] = -INFINITY;
        }
    }
    float m4[4];                                     // four independent max chains, then a tree
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int kb = c >> 1, v0 = (c & 1) * 8;
      m4[c] = max3(s[kb][v0], s[kb][v0 + 1], s[kb][v0 + 2]);
      m4[c] = max3(m4[c], s[kb][v0 + 3], s[kb][v0 + 4]);
      m4[c] = max3(m4[c], s[kb][v0 + 5], s[kb][v0 + 6]);
    }
    float mx = max3(max3(m4[0], s[0][7], s[0][15]), max3(m4[1], s[1][7], s[1][15]), fmaxf(m4[2], m4[3]));
    mx = pair_max(mx);
    const float m_new = fmaxf(m_run, mx * sc);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    const bool changed = m_new != m_run;
    m_run = m_new;
    // probabilities, rounded to bf16 in B-operand order; the row sum is taken over the rounded
    // values (the ones PV multiplies), two per instruction
    uint4 pf[2][2];
    float ps = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      float pv[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) pv[v] = __builtin_amdgcn_exp2f(fmaf(s[kb][v], sc, -m_new));
#pragma unroll
      for (int a2 = 0; a2 < 2; ++a2) {
        uint4 u;
        u.x = pack_bf16x2(pv[8 * a2 + 0], pv[8 * a2 + 1]);
        u.y = pack_bf16x2(pv[8 * a2 + 2], pv[8 * a2 + 3]);
        u.z = pack_bf16x2(pv[8 * a2 + 4], pv[8 * a2 + 5]);
        u.w = pack_bf16x2(pv[8 * a2 + 6], pv[8 * a2 + 7]);
        pf[kb][a2] = u;
        ps = pair_sum(u.x, ps);
        ps = pair_sum(u.y, ps);
        ps = pair_sum(u.z, ps);
        ps = pair_sum(u.w, ps);
      }
    }
    l_run = l_run * alpha + ps;
    if (__any(changed)) {                           // the running maximum rarely moves after the first tiles
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[mb][v] *= alpha;
    }
    typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
    // one LDS address per d-block; the (kb, a2, row group) part is a constant offset of the read
    lds_s16x4_ptr vptr[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) vptr[mb] = (lds_s16x4_ptr)(uintptr_t)(sbase + voff[mb]);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int a2 = 0; a2 < 2; ++a2)
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
          constexpr int ROWB = 256 / 8;                       // one key row in units of s16x4
          const s16x4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(vptr[mb] + (kb * 32 + a2 * 16) * ROWB);
          const s16x4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(vptr[mb] + (kb * 32 + a2 * 16 + 8) * ROWB);
          const uint2 u0 = __builtin_bit_cast(uint2, v0), u1 = __builtin_bit_cast(uint2, v1);
          uint4 vf;
          vf.x = u0.x; vf.y = u0.y; vf.z = u1.x; vf.w = u1.y;
          o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf),
                                                          __builtin_bit_cast(bf16x8_t, pf[kb][a2]), o[mb], 0, 0, 0);
        }
  };

  // ---- prologue: token ids of the first NS tiles, then the steady-state request pattern
  //      (ids of tile u + TOK_AHEAD, K/V tile u + NS - 1) for u = -(NS - 1) .. -1 ----
  for (int u = 0; u < NS; ++u) request_tokens(tile0 + u);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  for (int u = 0; u < NS - 1; ++u) {
    request_tokens(tile0 + u + NS);
    tile_tokens(tile0 + u, tokreg);
    request_rows(tile0 + u, 0, tokreg[0]);
    request_rows(tile0 + u, 1, tokreg[1]);
  }
  tile_tokens(tile0 + NS - 1, tokreg);

  // ---- tile segments of this wavefront ----
  const bool active = r0 < L;
  const int t_list_end = (list_len & 63) ? n_ctx_tiles - 1 : n_ctx_tiles;       // first masked context tile
  // chunk tile kt (keys 64 kt ..) is fully visible to the wave iff 64 kt + 63 <= r0, visible iff 64 kt <= r0 + 31
  const int t_diag = n_ctx_tiles + (active ? min(n_chunk_tiles, (r0 + 1) / 64) : 0);
  const int t_end = active ? n_ctx_tiles + min(n_chunk_tiles, (r0 + 31) / 64 + 1) : 0;
  using std::integral_constant;
  using std::true_type;
  using std::false_type;
  int t = tile0;
  if (active) {
    for (; t < min(t_list_end, tile1); ++t) tile(t, integral_constant<int, MASK_NONE>{}, true_type{});
    for (; t < min(n_ctx_tiles, tile1); ++t) tile(t, integral_constant<int, MASK_LIST_END>{}, true_type{});
    for (; t < min(t_diag, tile1); ++t) tile(t, integral_constant<int, MASK_NONE>{}, true_type{});
    for (; t < min(t_end, tile1); ++t) tile(t, integral_constant<int, MASK_CAUSAL>{}, true_type{});
  }
  for (; t < tile1; ++t) tile(t, integral_constant<int, MASK_NONE>{}, false_type{});
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the requests past the last tile

  // ---- epilogue ----
  uint16_t* Ob = reinterpret_cast<uint16_t*>(a.out) + (size_t)bi * L * D.Hq * d;
  const int qi = r0 + l32;
  const float lt = l_run + __shfl_xor(l_run, 32, 64);
  if (a.n_splits > 1) {
    // unnormalised O, running maximum and sum of this split: [seq][head][split][row][d + 2] fp32
    if (qi < L) {
      float* pr = a.part + ((((size_t)bi * D.Hq + head) * a.n_splits + split) * L + qi) * (d + 2);
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int a4 = 0; a4 < 4; ++a4)
          *reinterpret_cast<float4*>(pr + mb * 32 + 8 * a4 + 4 * hf) =
              make_float4(o[mb][4 * a4 + 0], o[mb][4 * a4 + 1], o[mb][4 * a4 + 2], o[mb][4 * a4 + 3]);
      if (hf == 0) { pr[d] = m_run; pr[d + 1] = lt; }
    }
    return;
  }
  if (a.part_mode == ATT_RETRIEVED) {
    // O = (w_a O_a + w_b O_b) / (w_a + w_b) with w = 2^(lse - max lse) (the log-sum-exp identity, log2 domain);
    // O_b = o / lt and lse_b = m_run + log2(lt), so w_b / lt = 2^(m_run - max). Every lane rewrites the
    // elements of O_a it reads. Without a retrieved key the first part stands as it is.
    if (qi < L) {
      const size_t rh = ((size_t)bi * L + qi) * D.Hq + head;
      const float la = a.lse_a[rh];
      if (lt > 0.f) {
        const float la2 = la * 1.4426950408889634f, lb2 = m_run + log2f(lt);
        const float mx = fmaxf(la2, lb2);
        const float wa = __builtin_amdgcn_exp2f(la2 - mx), wb = __builtin_amdgcn_exp2f(lb2 - mx);
        const float inv = 1.f / (wa + wb);
        const float fa = wa * inv, fb = __builtin_amdgcn_exp2f(m_run - mx) * inv;
        uint16_t* orow = Ob + ((size_t)qi * D.Hq + head) * d;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int a4 = 0; a4 < 4; ++a4) {
            uint2* p = reinterpret_cast<uint2*>(orow + mb * 32 + 8 * a4 + 4 * hf);
            const uint2 ua = *p;
            uint2 u;
            u.x = pack_bf16x2(fa * __uint_as_float(ua.x << 16) + fb * o[mb][4 * a4 + 0],
                              fa * __uint_as_float(ua.x & 0xFFFF0000u) + fb * o[mb][4 * a4 + 1]);
            u.y = pack_bf16x2(fa * __uint_as_float(ua.y << 16) + fb * o[mb][4 * a4 + 2],
                              fa * __uint_as_float(ua.y & 0xFFFF0000u) + fb * o[mb][4 * a4 + 3]);
            *p = u;
          }
        if (a.lse && hf == 0) a.lse[rh] = (mx + log2f(wa + wb)) * 0.6931471805599453f;
      } else if (a.lse && hf == 0) {
        a.lse[rh] = la;
      }
    }
    return;
  }
  if (qi < L) {
    const float inv = 1.f / lt;
    uint16_t* orow = Ob + ((size_t)qi * D.Hq + head) * d;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int a4 = 0; a4 < 4; ++a4) {
        uint2 u;
        u.x = pack_bf16x2(o[mb][4 * a4 + 0] * inv, o[mb][4 * a4 + 1] * inv);
        u.y = pack_bf16x2(o[mb][4 * a4 + 2] * inv, o[mb][4 * a4 + 3] * inv);
        *reinterpret_cast<uint2*>(orow + mb * 32 + 8 * a4 + 4 * hf) = u;
      }
    if (a.lse && hf == 0)
      a.lse[((size_t)bi * L + qi) * D.Hq + head] = (m_run + log2f(lt)) * 0.6931471805599453f;
  }
}

// ---- merge of the splits of a short query block: O = sum_s w_s O_s / sum_s w_s l_s,
//      w_s = 2^(m_s - max m) (the log-sum-exp identity), one workgroup per (row, head, sequence) ----
__global__ __launch_bounds__(128) void attend_merge_kernel(AttArgs a) {
  const Dims& D = a.D;
  const int qi = blockIdx.x, head = blockIdx.y, bi = blockIdx.z, d = 128, L = a.n_q, c = threadIdx.x;
  const float* pr = a.part + ((size_t)bi * D.Hq + head) * a.n_splits * L * (d + 2);
  float mmax = -1e30f;
  for (int s = 0; s < a.n_splits; ++s) mmax = fmaxf(mmax, pr[((size_t)s * L + qi) * (d + 2) + d]);
  float acc = 0.f, l = 0.f;
  for (int s = 0; s < a.n_splits; ++s) {
    const float* q = pr + ((size_t)s * L + qi) * (d + 2);
    const float w = __builtin_amdgcn_exp2f(q[d] - mmax);
    acc = fmaf(w, q[c], acc);
    l = fmaf(w, q[d + 1], l);
  }
  uint16_t* orow = reinterpret_cast<uint16_t*>(a.out) + (((size_t)bi * L + qi) * D.Hq + head) * d;
  orow[c] = f32_to_bf16(acc / l);
  if (a.lse && c == 0) a.lse[((size_t)bi * L + qi) * D.Hq + head] = (mmax + log2f(l)) * 0.6931471805599453f;
}

// ---- one query row per sequence (decode, G <= 4): keys across wavefronts, nothing staged in LDS ----
// The step reads every K and V row of the context once and does next to no arithmetic, so the kernel is
// built to keep loads in flight: a workgroup is four wavefronts that walk disjoint runs of 16-key groups of
// one (sequence, KV head, split), each on its own (no barrier in the loop); up to three workgroups fit a
// compute unit. Per group a lane fetches 16-byte pieces straight into matrix-core operand order:
//   S^T = K Q^T by v_mfma_f32_16x16x32_bf16: A = 16 keys x 32 d (lane: key lane % 16, d-piece lane / 16),
//   B = Q^T with the heads of the group in columns 0 .. G - 1 and zeros beyond; the result leaves keys
//   4 (lane / 16) + j, j < 4, of head lane % 16 in lane's four registers;
//   O += P V on the vector ALU: a lane owns 8 d-columns (lane % 16) of the 4 keys of its lane group, fetches
//   their V pieces (one 16-byte load per key) and the 4 x G probabilities from the lanes that hold them.
// The running maximum is per head (lane column); the rescale factor of every head reaches all lanes by a
// lane read. Rows of group g + 1 and token ids of group g + 2 are in flight while group g is used. At the
// end the four lane groups' partial O and sums are added, the four wavefronts merge through LDS, and the
// workgroup writes one partial result in the layout attend_merge_kernel reads.
constexpr int DEC_WAVES = 4;
template <int G>
__global__ __launch_bounds__(64 * DEC_WAVES, 3) void attend_decode_kernel(AttArgs a) {
  constexpr int d = 128;
  __shared__ float wpart[DEC_WAVES][G][d + 2];
  const Dims& D = a.D;
  const int split = blockIdx.x, h = blockIdx.y, bi = blockIdx.z;
  const int seq = a.bp.seq[bi], c0 = a.bp.c0[bi];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kl = lane & 15, grp = lane >> 4;
  const int slot = slot_of(D, a.layer, seq, h);
  const unsigned char* Kb = reinterpret_cast<const unsigned char*>(a.k_arena) + arena_off(D, slot) * 2;
  const unsigned char* Vb = reinterpret_cast<const unsigned char*>(a.v_arena) + arena_off(D, slot) * 2;
  const int list_len = a.st.meta[(size_t)slot * META_WORDS + META_LIST_LEN];
  const int32_t* list = a.st.row_list + (size_t)slot * D.list_cap;
  const int n_keys = list_len + 1;                  // the context list and the token itself
  const int crow0 = chunk_tok_row(D, c0, c0);
  const int n_groups = (n_keys + 15) >> 4;
  const int workers = a.n_splits * DEC_WAVES, w = split * DEC_WAVES + wave;
  const int gpw = (n_groups + workers - 1) / workers;
  const int g_begin = min(w * gpw, n_groups), g_end = min(g_begin + gpw, n_groups);

  // B operand: Q^T, head kl of the group in column kl
  uint4 qf[4];
  {
    const uint16_t* qrow = reinterpret_cast<const uint16_t*>(a.q) + ((size_t)bi * D.Hq + (size_t)h * G + min(kl, G - 1)) * d;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      qf[kk] = *reinterpret_cast<const uint4*>(qrow + kk * 32 + grp * 8);
      if (kl >= G) qf[kk] = make_uint4(0u, 0u, 0u, 0u);
    }
  }
  // Tokens of the keys this lane fetches in group g: its K row (key kl) and its four V rows (keys
  // 4 grp + j). Indices are clamped to the last key, so masked keys read a valid row.
  struct Toks { int k, v[4]; };
  auto load_tokens = [&](int g, Toks& t) __attribute__((always_inline)) {
    const int rk = min(g * 16 + kl, n_keys - 1);
    t.k = rk < list_len ? list[rk] : crow0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int rv = min(g * 16 + 4 * grp + j, n_keys - 1);
      t.v[j] = rv < list_len ? list[rv] : crow0;
    }
  };
  auto load_rows = [&](const Toks& t, uint4 (&kf)[4], uint4 (&vf)[4]) __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      kf[kk] = *reinterpret_cast<const uint4*>(Kb + ((size_t)t.k << 8) + kk * 64 + grp * 16);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      vf[j] = *reinterpret_cast<const uint4*>(Vb + ((size_t)t.v[j] << 8) + kl * 16);
  };

  float o[G][8];
#pragma unroll
  for (int hh = 0; hh < G; ++hh)
#pragma unroll
    for (int c = 0; c < 8; ++c) o[hh][c] = 0.f;
  float m_run = -1e30f, l_lane = 0.f;               // of head kl (log2 domain); the sum over this lane's keys only
  const float sc = 1.4426950408889634f / sqrtf((float)d);

  auto compute = [&](int g, const uint4 (&kf)[4], const uint4 (&vf)[4]) __attribute__((always_inline)) {
    f32x4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf[kk]),
                                                  __builtin_bit_cast(bf16x8_t, qf[kk]), s, 0, 0, 0);
    float sv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) sv[j] = (g * 16 + 4 * grp + j < n_keys) ? s[j] * sc : -INFINITY;
    float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    const bool moved = __any(kl < G && m_new != m_run);
    m_run = m_new;
    float pv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) pv[j] = __builtin_amdgcn_exp2f(sv[j] - m_new);
    l_lane = l_lane * alpha + ((pv[0] + pv[1]) + (pv[2] + pv[3]));
    if (moved) {                                    // the running maxima rarely move after the first groups
#pragma unroll
      for (int hh = 0; hh < G; ++hh) {
        const float ah = __shfl(alpha, hh, 64);     // lane hh holds head hh's factor
#pragma unroll
        for (int c = 0; c < 8; ++c) o[hh][c] *= ah;
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint4 u = vf[j];
      float vv[8];
      vv[0] = __uint_as_float(u.x << 16); vv[1] = __uint_as_float(u.x & 0xFFFF0000u);
      vv[2] = __uint_as_float(u.y << 16); vv[3] = __uint_as_float(u.y & 0xFFFF0000u);
      vv[4] = __uint_as_float(u.z << 16); vv[5] = __uint_as_float(u.z & 0xFFFF0000u);
      vv[6] = __uint_as_float(u.w << 16); vv[7] = __uint_as_float(u.w & 0xFFFF0000u);
#pragma unroll
      for (int hh = 0; hh < G; ++hh) {
        const float ph = __shfl(pv[j], (lane & 48) | hh, 64);   // key 4 grp + j of head hh
#pragma unroll
        for (int c = 0; c < 8; ++c) o[hh][c] = fmaf(ph, vv[c], o[hh][c]);
      }
    }
  };

  // Rows of group g + 1 and tokens of group g + 2 are requested before group g is used; the two
  // row buffers alternate by name so that they stay in registers.
  uint4 ka[4], va[4], kb[4], vb[4];
  Toks t0, t1;
  int g = g_begin;
  if (g < g_end) {
    load_tokens(g, t0);
    load_rows(t0, ka, va);
    if (g + 1 < g_end) load_tokens(g + 1, t1);
  }
  while (g < g_end) {
    if (g + 1 < g_end) load_rows(t1, kb, vb);
    if (g + 2 < g_end) load_tokens(g + 2, t0);
    compute(g, ka, va);
    if (++g >= g_end) break;
    if (g + 1 < g_end) load_rows(t0, ka, va);
    if (g + 2 < g_end) load_tokens(g + 2, t1);
    compute(g, kb, vb);
    ++g;
  }
  // the four lane groups hold disjoint keys: add their partial results
  l_lane += __shfl_xor(l_lane, 16, 64);
  l_lane += __shfl_xor(l_lane, 32, 64);
#pragma unroll
  for (int hh = 0; hh < G; ++hh)
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      float v = o[hh][c];
      v += __shfl_xor(v, 16, 64);
      v += __shfl_xor(v, 32, 64);
      o[hh][c] = v;
    }
  if (grp == 0) {
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
      for (int c = 0; c < 8; ++c) wpart[wave][hh][kl * 8 + c] = o[hh][c];
    if (kl < G) { wpart[wave][kl][d] = m_run; wpart[wave][kl][d + 1] = l_lane; }
  }
  __syncthreads();
  // merge of the four wavefronts; one partial result per (head, split): unnormalised O, maximum, sum
  for (int idx = threadIdx.x; idx < G * d; idx += 64 * DEC_WAVES) {
    const int hh = idx / d, c = idx - hh * d;
    float mmax = -1e30f;
#pragma unroll
    for (int ww = 0; ww < DEC_WAVES; ++ww) mmax = fmaxf(mmax, wpart[ww][hh][d]);
    float acc = 0.f, l = 0.f;
#pragma unroll
    for (int ww = 0; ww < DEC_WAVES; ++ww) {
      const float wgt = __builtin_amdgcn_exp2f(wpart[ww][hh][d] - mmax);
      acc = fmaf(wgt, wpart[ww][hh][c], acc);
      l = fmaf(wgt, wpart[ww][hh][d + 1], l);
    }
    float* pr = a.part + (((size_t)bi * D.Hq + (size_t)h * G + hh) * a.n_splits + split) * (d + 2);
    pr[c] = acc;
    if (c == 0) { pr[d] = mmax; pr[d + 1] = l; }
  }
}

// ---- first part of a two-part step: its token list ----
// initial | window tokens of every sequence of the batch, padded with token 0 to whole tiles
__global__ __launch_bounds__(256) void local_list_kernel(Dims D, BatchPos bp, int32_t* loclist, int loc_cap) {
  const int bi = blockIdx.y, c0 = bp.c0[bi];
  const int n_init = min(D.n_sink, c0), w0 = max(n_init, c0 - D.window), len = n_init + c0 - w0;
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r < loc_cap) loclist[(size_t)bi * loc_cap + r] = r < n_init ? r : (r < len ? window_tok_row(D, w0 + r - n_init) : 0);
}

// ---- fp32 kernel: one wavefront per (query row, head); keys across lanes ----
template <int DT>
__global__ __launch_bounds__(64) void attend_simple_kernel(AttArgs a) {
  typedef typename Elt<DT>::type T;
  __shared__ float qs[128];
  __shared__ float ps[64];
  __shared__ int toks[64];
  const Dims& D = a.D;
  const int qi = blockIdx.x, head = blockIdx.y, bi = blockIdx.z;
  const int h = head / D.G, d = D.d, per = d / 64;
  const int seq = a.bp.seq[bi], c0 = a.bp.c0[bi], L = a.n_q;
  const int lane = threadIdx.x;
  const int slot = slot_of(D, a.layer, seq, h);
  const T* Kb = reinterpret_cast<const T*>(a.k_arena) + arena_off(D, slot);
  const T* Vb = reinterpret_cast<const T*>(a.v_arena) + arena_off(D, slot);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int list_len = meta[META_LIST_LEN];
  const int32_t* list = a.st.row_list + (size_t)slot * D.list_cap;
  const T* qrow = reinterpret_cast<const T*>(a.q) + (((size_t)bi * L + qi) * D.Hq + head) * d;
  for (int c = lane; c < d; c += 64) qs[c] = Elt<DT>::to_f32(qrow[c]);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)d);
  const int n_keys = list_len + qi + 1;
  float m_run = -1e30f, l_run = 0.f, o0 = 0.f, o1 = 0.f;
  for (int k0 = 0; k0 < n_keys; k0 += 64) {
    const int k = k0 + lane;
    int tok = -1;
    if (k < list_len) tok = list[k];
    else if (k < n_keys) tok = chunk_tok_row(D, c0, c0) + (k - list_len);
    float z = -INFINITY;
    if (tok >= 0) {
      const T* krow = Kb + (size_t)tok * d;
      float acc = 0.f;
      for (int c = 0; c < d; ++c) acc = fmaf(qs[c], Elt<DT>::to_f32(krow[c]), acc);
      z = acc * scale;
    }
    float mx = z;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = expf(m_run - m_new);
    const float pz = expf(z - m_new);
    float sum = pz;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    l_run = l_run * alpha + sum;
    m_run = m_new;
    __syncthreads();
    ps[lane] = pz;
    toks[lane] = tok;
    __syncthreads();
    o0 *= alpha; o1 *= alpha;
    const int cnt = min(64, n_keys - k0);
    for (int kk = 0; kk < cnt; ++kk) {
      const int tk = toks[kk];
      if (tk < 0) continue;
      const T* vrow = Vb + (size_t)tk * d + lane * per;
      o0 = fmaf(ps[kk], Elt<DT>::to_f32(vrow[0]), o0);
      if (per == 2) o1 = fmaf(ps[kk], Elt<DT>::to_f32(vrow[1]), o1);
    }
  }
  T* orow = reinterpret_cast<T*>(a.out) + (((size_t)bi * L + qi) * D.Hq + head) * d + lane * per;
  const float inv = 1.f / l_run;
  orow[0] = Elt<DT>::from_f32(o0 * inv);
  if (per == 2) orow[1] = Elt<DT>::from_f32(o1 * inv);
  if (a.lse && lane == 0) a.lse[((size_t)bi * L + qi) * D.Hq + head] = m_run + logf(l_run);
}

// ---- standalone gather: K/V rows of the context list into packed buffers ----
struct GatherArgs { Dims D; DevState st; const void* k_arena; const void* v_arena; int layer, seq;
                    void* k_packed; void* v_packed; int32_t* n_tokens; };

constexpr int GATHER_ROWS = 4;
__global__ __launch_bounds__(256) void gather_pack_kernel(GatherArgs a) {
  const Dims& D = a.D;
  const int h = blockIdx.y;
  const int slot = slot_of(D, a.layer, a.seq, h);
  const int32_t* meta = a.st.meta + (size_t)slot * META_WORDS;
  const int list_len = meta[META_LIST_LEN];
  const int32_t* list = a.st.row_list + (size_t)slot * D.list_cap;
  const int row16 = D.d * D.elt / 16;                        // 16-byte pieces per row
  const int rows_per_pass = 256 / row16;
  const int r_in = threadIdx.x / row16, piece = threadIdx.x - r_in * row16;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4* Kb = reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(a.k_arena) + arena_off(D, slot) * D.elt);
  const u32x4* Vb = reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(a.v_arena) + arena_off(D, slot) * D.elt);
  u32x4* Kp = reinterpret_cast<u32x4*>(a.k_packed) + (size_t)h * D.list_cap * row16;
  u32x4* Vp = reinterpret_cast<u32x4*>(a.v_packed) + (size_t)h * D.list_cap * row16;
  // GATHER_ROWS rows per thread and trip: the token ids first, then all the row pieces (2 x GATHER_ROWS independent
  // 16-byte loads in flight per lane), then the stores, which nothing reads again soon (non-temporal)
  const int stride = gridDim.x * rows_per_pass;
  for (int r0 = blockIdx.x * rows_per_pass + r_in; r0 < list_len; r0 += GATHER_ROWS * stride) {
    int tok[GATHER_ROWS];
#pragma unroll
    for (int u = 0; u < GATHER_ROWS; ++u) tok[u] = list[min(r0 + u * stride, list_len - 1)];
    u32x4 kv[GATHER_ROWS], vv[GATHER_ROWS];
#pragma unroll
    for (int u = 0; u < GATHER_ROWS; ++u) {
      kv[u] = Kb[(size_t)tok[u] * row16 + piece];
      vv[u] = Vb[(size_t)tok[u] * row16 + piece];
    }
#pragma unroll
    for (int u = 0; u < GATHER_ROWS; ++u) {
      const int r = r0 + u * stride;
      if (r < list_len) {
        __builtin_nontemporal_store(kv[u], Kp + (size_t)r * row16 + piece);
        __builtin_nontemporal_store(vv[u], Vp + (size_t)r * row16 + piece);
      }
    }
  }
  if (a.n_tokens && blockIdx.x == 0 && threadIdx.x == 0) a.n_tokens[h] = list_len;
}

// ---- how a launch splits the key range of a short query block, and what its partial results need ----
// kind: 0 = no partial results, 1 = the one-token kernel, 2 = the matrix-core kernel with splits
static int attend_split_count(const Dims& D, int seq_count, int n_q, int n_cus, int* kind) {
  *kind = 0;
  if (!attend_on_matrix_cores(D) || n_q > ATT_SPLIT_MAX_ROWS) return 1;
  if (n_q == 1 && D.G <= 4) {
    // decode: two workgroups per compute unit (measured best at 16 sequences x 8 KV heads: 67 us against
    // 70 .. 81 us with 3 .. 16 splits; the step runs at the rate of a plain copy either way)
    const int slots = D.Hkv * seq_count;
    const int ns = (2 * n_cus) / slots;
    *kind = 1;
    return ns > ATT_MAX_SPLITS ? ATT_MAX_SPLITS : (ns < 1 ? 1 : ns);
  }
  // a short query block on few workgroups: split the key range so that every compute unit streams a
  // share of it; the partial results are merged by a second kernel
  const int HG = D.G < 4 ? D.G : 4;
  const int blocks = D.Hkv * (D.G / HG) * seq_count;
  if (blocks >= 256) return 1;
  const int ns = 256 / blocks;
  if (ns <= 1) return 1;
  *kind = 2;
  return ns > ATT_MAX_SPLITS ? ATT_MAX_SPLITS : ns;
}

static hipError_t device_cus(int* n_cus) {
  static int cached = 0;
  if (cached == 0) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cached, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) { cached = 0; return e; }
  }
  *n_cus = cached;
  return hipSuccess;
}

size_t attend_partial_bytes(const Dims& D, int seq_count, int n_q, int n_cus) {
  int kind = 0;
  const int ns = attend_split_count(D, seq_count, n_q, n_cus, &kind);
  if (kind == 0) return 0;
  return (size_t)seq_count * D.Hq * ns * (kind == 1 ? 1 : n_q) * (D.d + 2) * sizeof(float);
}

// ---- partial results for callers that bring no buffer ----
// One array per GPU, held from the moment the library is loaded until the process ends. In host code the
// array's name is only a handle for hipGetSymbolAddress; the address the kernels get is the one that call
// returns, looked up once per device with that device current.
static __device__ __align__(256) unsigned char scratch[ATT_STATIC_SCRATCH_BYTES];

hipError_t attend_static_scratch(float** ptr) {
  constexpr int MAX_DEVICES = 64;
  static void* per_device[MAX_DEVICES] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (!per_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    per_device[dev] = p;
  }
  *ptr = static_cast<float*>(per_device[dev]);
  return hipSuccess;
}

hipError_t launch_attend(const Dims& D, const DevState& st, const void* k_arena, const void* v_arena,
                         const void* q, int layer, const BatchPos& bp, int seq_count, int n_q,
                         void* out, float* lse, int stages, float* part, int part_mode, const int32_t* loclist,
                         int loc_cap, const float* lse_a, hipStream_t s, hipEvent_t t_begin, hipEvent_t t_end) {
  if ((t_begin == nullptr) != (t_end == nullptr)) return hipErrorInvalidValue;
  AttArgs a;
  a.D = D; a.st = st; a.k_arena = k_arena; a.v_arena = v_arena; a.q = q; a.out = out; a.lse = lse;
  a.layer = layer; a.seq_count = seq_count; a.n_q = n_q; a.bp = bp;
  a.n_splits = 1; a.part = part;
  a.part_mode = part_mode; a.loclist = loclist; a.loc_cap = loc_cap; a.lse_a = lse_a;
  if (part_mode == ATT_RETRIEVED && !lse_a) return hipErrorInvalidValue;
  const bool mfma_ok = attend_on_matrix_cores(D);
  if (part_mode != ATT_ALL && (!mfma_ok || n_q <= ATT_SPLIT_MAX_ROWS)) return hipErrorInvalidValue;
  int n_cus = 0, kind = 0;
  if (hipError_t e = device_cus(&n_cus); e != hipSuccess) return e;
  const int ns_short = (part && part_mode == ATT_ALL) ? attend_split_count(D, seq_count, n_q, n_cus, &kind) : 1;
  if (kind == 1) {
    a.n_splits = ns_short;
    dim3 g(a.n_splits, D.Hkv, seq_count);
    if (t_begin) { if (hipError_t e = hipEventRecord(t_begin, s); e != hipSuccess) return e; }
    if (D.G == 4)      attend_decode_kernel<4><<<g, 64 * DEC_WAVES, 0, s>>>(a);
    else if (D.G == 2) attend_decode_kernel<2><<<g, 64 * DEC_WAVES, 0, s>>>(a);
    else               attend_decode_kernel<1><<<g, 64 * DEC_WAVES, 0, s>>>(a);
    attend_merge_kernel<<<dim3(1, D.Hq, seq_count), 128, 0, s>>>(a);
    if (t_end) { if (hipError_t e = hipEventRecord(t_end, s); e != hipSuccess) return e; }
    return hipGetLastError();
  }
  if (mfma_ok) {
    const int HG = D.G < 4 ? D.G : 4;
    const int gpk = D.G / HG;
    constexpr int NW = ATT_NW;
    const int RPB = 32 * (NW / HG);
    dim3 g(D.Hkv * gpk, (n_q + RPB - 1) / RPB, seq_count);
    if (kind == 2) {
      a.n_splits = ns_short;
      g.y = a.n_splits;
    }
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_bf16_kernel<NW, 4>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, att_lds_bytes(4, NW));
      if (e != hipSuccess) return e;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_bf16_kernel<NW, 3>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, att_lds_bytes(3, NW));
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    if (t_begin) {
      // the events ride in the kernel's own dispatch; with a merge behind it the end is recorded after that
      const hipEvent_t stop = a.n_splits > 1 ? nullptr : t_end;
      if (stages == 3)
        hipExtLaunchKernelGGL((attend_bf16_kernel<NW, 3>), g, dim3(64 * NW), (uint32_t)att_lds_bytes(3, NW), s, t_begin, stop, 0, a);
      else
        hipExtLaunchKernelGGL((attend_bf16_kernel<NW, 4>), g, dim3(64 * NW), (uint32_t)att_lds_bytes(4, NW), s, t_begin, stop, 0, a);
    } else if (stages == 3) {
      attend_bf16_kernel<NW, 3><<<g, 64 * NW, att_lds_bytes(3, NW), s>>>(a);
    } else {
      attend_bf16_kernel<NW, 4><<<g, 64 * NW, att_lds_bytes(4, NW), s>>>(a);
    }
    if (a.n_splits > 1) {
      attend_merge_kernel<<<dim3(n_q, D.Hq, seq_count), 128, 0, s>>>(a);
      if (t_end) { if (hipError_t e = hipEventRecord(t_end, s); e != hipSuccess) return e; }
    }
  } else {
    dim3 g(n_q, D.Hq, seq_count);
    if (t_begin) { if (hipError_t e = hipEventRecord(t_begin, s); e != hipSuccess) return e; }
    if (D.dtype == LTRI_BF16) attend_simple_kernel<LTRI_BF16><<<g, 64, 0, s>>>(a);
    else                      attend_simple_kernel<LTRI_F32><<<g, 64, 0, s>>>(a);
    if (t_end) { if (hipError_t e = hipEventRecord(t_end, s); e != hipSuccess) return e; }
  }
  return hipGetLastError();
}

bool attend_on_matrix_cores(const Dims& D) {
  return D.dtype == LTRI_BF16 && D.d == 128 && (D.G == 1 || D.G == 2 || D.G % 4 == 0);
}

hipError_t launch_local_list(const Dims& D, const BatchPos& bp, int seq_count, int32_t* loclist, int loc_cap,
                             hipStream_t s) {
  local_list_kernel<<<dim3((loc_cap + 255) / 256, seq_count), 256, 0, s>>>(D, bp, loclist, loc_cap);
  return hipGetLastError();
}

hipError_t launch_gather_pack(const Dims& D, const DevState& st, const void* k_arena, const void* v_arena,
                              int layer, int seq, void* k_packed, void* v_packed, int32_t* n_tokens,
                              hipStream_t s) {
  GatherArgs a{D, st, k_arena, v_arena, layer, seq, k_packed, v_packed, n_tokens};
  const int row16 = D.d * D.elt / 16;
  const int rows_per_pass = 256 / row16;
  int gx = (D.list_cap + rows_per_pass * GATHER_ROWS - 1) / (rows_per_pass * GATHER_ROWS);
  if (gx < 1) gx = 1;
  dim3 g(gx, D.Hkv);
  gather_pack_kernel<<<g, 256, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace ltri
