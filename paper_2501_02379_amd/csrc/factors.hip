// Factor refresh: {U^(n)} <- TuckerFactors(R_L, r), third line of the refresh branch of
// Algorithm 1, as HOSVD (appendix "Implementation": truncated SVD of every mode-n unfolding).
// The left singular vectors of the unfolding R_L(n) are the eigenvectors of the Hermitian
// mode-n Gram matrix A_n = R_L(n) R_L(n)^H, so the refresh is
//   (1) A_n for every compressed mode, accumulated in float64 on the f64 matrix cores, with
//       R_L = G - Sparse(G, Omega) formed on load from the support bitmask, and
//   (2) an eigen-solve of each A_n in float64 (one workgroup per mode) for its r_n leading
//       eigenvectors, written eigenvalue-descending with the phase of every column fixed
//       (largest-modulus entry real and positive): tridiagonalisation + bisection + inverse
//       iteration for extents up to 128, cyclic Jacobi for clustered spectra and larger extents.
// float64 is used because Adam in core space is not invariant to the basis inside the subspace:
// noise-like gradients have relative eigenvalue gaps near 1e-4, and float32 accumulation error
// divided by such a gap would move the individual eigenvectors far more than the update tolerates.
#include <type_traits>

#include "device_common.h"

namespace tgrad {

namespace {

typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int kSuper = 128;          // rows of the output handled by one workgroup, per side
constexpr int kTC = 16;              // tensor columns staged per tile
constexpr int kRowD = 4 * kTC + 2;   // doubles per staged row: 4 per element + a pad of 16 bytes (conflict-free reads)
constexpr int kGramThreads = 1024;   // 16 wavefronts: a 4 x 4 grid of 32 x 32 output blocks

// Gram of the tensor viewed as (A, In, B): gram[i, j] = sum_{a, b} x[a, i, b] conj(x[a, j, b]).
// Real embedding on v_mfma_f64_16x16x4f64 (K = 4 = two tensor columns x {re, im}):
//   Re[i, j] = sum xr_i xr_j + xi_i xi_j      -> A operand (xr_i | xi_i),  B operand (xr_j | xi_j)
//   Im[i, j] = sum xi_i xr_j - xr_i xi_j      -> A operand (xi_i | -xr_i), B operand (xr_j | xi_j)
// Operand lanes: A[i = lane % 16][k = lane / 16], B[k = lane / 16][j = lane % 16];
// result: register r of lane l holds D[4 r + l / 16][l % 16].
// The matrix is Hermitian, so only its lower triangle is computed: a workgroup owns one 128 x 128
// super block (si >= sj) of one chunk of tensor columns, cut into 16 x 16 matrix-core tiles - all 64
// of them off the diagonal, the 36 on or below it on the diagonal - dealt round-robin to its 16
// wavefronts (tile t to wavefront t % 16: 9 tiles per SIMD in the diagonal case).  The next
// 16 columns are fetched into registers while the current ones are in the matrix cores.
// A staged element is converted to float64 once, when it is committed to LDS, and stored as the four
// operands it can be asked for: (xr, xi, xi, -xr).  The f64 matrix instructions run on the SIMD's
// vector ALU; a conversion and a select per operand fetch in the inner loop (each element is an
// operand of up to 8 tiles) took as many of its cycles as the matrix instructions themselves.
constexpr int kGramMaxTiles = 4;     // tiles per wavefront: 64 / 16

template <int DT>
__global__ __launch_bounds__(kGramThreads) void k_gram(const void* __restrict__ x,
                                                        const uint32_t* __restrict__ mask, int64_t A,
                                                        int In, int64_t B, int64_t cols_per_chunk,
                                                        double* __restrict__ partials) {
  extern __shared__ double sG[];
  double* sI = sG;                                    // [row][column][xr, xi, xi, -xr]
  double* sJ = sG + kSuper * kRowD;
  const int nsup = (In + kSuper - 1) / kSuper;
  const int si = blockIdx.y / nsup, sj = blockIdx.y % nsup;
  if (si < sj) return;                                // upper super blocks: mirrored by the reduction
  const bool diag = si == sj;
  const int64_t J = A * B;
  const int64_t c_begin = (int64_t)blockIdx.x * cols_per_chunk;
  const int64_t c_end = c_begin + cols_per_chunk < J ? c_begin + cols_per_chunk : J;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int part = (lane >> 4) & 1;
  const int ccol = lane >> 5;
  const int lrow = lane & 15;
  const int rows_i = In - si * kSuper < kSuper ? In - si * kSuper : kSuper;   // rows present in the two
  const int rows_j = In - sj * kSuper < kSuper ? In - sj * kSuper : kSuper;   // super blocks

  // this wavefront's tiles: slot k holds tile t = wave + 16 k (static slots: no dynamic indexing)
  int ti[kGramMaxTiles], tj[kGramMaxTiles];
  bool mine[kGramMaxTiles];
  const int ntl = diag ? 36 : 64;
#pragma unroll
  for (int k = 0; k < kGramMaxTiles; ++k) {
    const int t = wave + 16 * k;
    int a = 0, b = 0;
    if (diag) {
      a = (int)((sqrtf(8.f * (float)t + 1.f) - 1.f) * 0.5f);
      while (a * (a + 1) / 2 > t) --a;
      while ((a + 1) * (a + 2) / 2 <= t) ++a;
      b = t - a * (a + 1) / 2;
    } else {
      a = t >> 3;
      b = t & 7;
    }
    mine[k] = t < ntl && 16 * a < rows_i && 16 * b < rows_j;   // tiles of absent rows hold zeros: skipped
    ti[k] = mine[k] ? a : 0;
    tj[k] = mine[k] ? b : 0;
  }

  v4d accRe[kGramMaxTiles], accIm[kGramMaxTiles];
#pragma unroll
  for (int k = 0; k < kGramMaxTiles; ++k) {
    accRe[k] = (v4d){0., 0., 0., 0.};
    accIm[k] = (v4d){0., 0., 0., 0.};
  }

  // A thread stages elements e = tid + u * 1024 (u < kPer) of a tile: row il, column cl.  Which ones
  // they are does not depend on the tile, so everything that can be is computed once: the LDS slot,
  // the tensor offset of (row, cl) inside a tile, and whether the row exists.
  constexpr int kPer = kSuper * kTC / kGramThreads;   // 2 elements per thread and side
  int e_cl[kPer], e_lds[kPer];
  int64_t e_offI[kPer], e_offJ[kPer];                 // (row * B + cl) for the row side / the column side
  bool e_okI[kPer], e_okJ[kPer];
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int e = tid + u * kGramThreads;
    int il, cl;
    if (B == 1) {                                     // rows are the fastest index in memory
      il = e % kSuper;
      cl = e / kSuper;
    } else {                                          // columns b are the fastest index
      il = e / kTC;
      cl = e % kTC;
    }
    e_cl[u] = cl;
    e_lds[u] = il * kRowD + 4 * cl;
    e_okI[u] = si * kSuper + il < In;
    e_okJ[u] = sj * kSuper + il < In;
    e_offI[u] = (int64_t)(si * kSuper + il) * B + cl;
    e_offJ[u] = (int64_t)(sj * kSuper + il) * B + cl;
  }
  // Column c = c0 + cl of the unfolding is tensor index (a, b) = (c / B, c % B); with (a0, b0) those
  // of the tile's first column (kept up to date by the caller) the element (row i, column c) lies at
  //   (a0 In + i) B + b0 + cl            if b0 + cl < B,
  //   ... + (In - 1) B                   if the column has wrapped into the next a (at most once
  //                                      per tile when B >= 16; smaller B take the general form).
  // A 64-bit division per fetched element would cost the vector ALU - which the f64 matrix
  // instructions also run on - more cycles than the tile's matrix instructions.
  const int64_t wrap_add = (int64_t)(In - 1) * B;
  auto fetch = [&](bool row_ok, int64_t off, int cl, int64_t c0, int64_t a0, int64_t b0) -> float2 {
    float2 v = make_float2(0.f, 0.f);
    if (row_ok && c0 + cl < c_end) {
      int64_t idx;
      if (B >= kTC) {
        idx = a0 * In * B + b0 + off + (b0 + cl >= B ? wrap_add : (int64_t)0);
      } else {                                        // tiny trailing extent: b0 + cl < 32
        const uint32_t q = (uint32_t)(b0 + cl) / (uint32_t)B;
        idx = a0 * In * B + b0 + off + (int64_t)q * wrap_add;
      }
      // both loads are issued together (a load that waits for the mask bit would double the latency)
      const uint32_t mw = mask ? mask[idx >> 5] : 0u;
      const float2 xv = load_elem<DT>(x, idx);
      if (!((mw >> (idx & 31)) & 1u)) v = xv;
    }
    return v;
  };

  float2 preI[kPer], preJ[kPer];                      // next tile of the row side / the column side
  int64_t pa0 = c_begin / B, pb0 = c_begin - pa0 * B; // of the tile being fetched (workgroup-uniform)
  auto next_tile = [&]() {                            // (a0, b0) of the tile kTC columns further on
    pb0 += kTC;
    if (B >= kTC) {
      if (pb0 >= B) { pb0 -= B; pa0 += 1; }
    } else {
      const uint32_t q = (uint32_t)pb0 / (uint32_t)B;
      pa0 += q;
      pb0 -= (int64_t)q * B;
    }
  };
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    preI[u] = fetch(e_okI[u], e_offI[u], e_cl[u], c_begin, pa0, pb0);
    preJ[u] = diag ? make_float2(0.f, 0.f) : fetch(e_okJ[u], e_offJ[u], e_cl[u], c_begin, pa0, pb0);
  }

  // pre -> one staged tile (row side into dI; column side into dJ when the super block is off the diagonal)
  auto commit = [&](double* dI, double* dJ) {
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      {
        const double xr = (double)preI[u].x, xi = (double)preI[u].y;
        double2* d = reinterpret_cast<double2*>(dI + e_lds[u]);
        d[0] = make_double2(xr, xi);
        d[1] = make_double2(xi, -xr);
      }
      if (!diag) {
        const double xr = (double)preJ[u].x, xi = (double)preJ[u].y;
        *reinterpret_cast<double2*>(dJ + e_lds[u]) = make_double2(xr, xi);
      }
    }
  };
  auto prefetch = [&](int64_t c0) {                   // the tile that starts at column c0 -> pre
    next_tile();
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      preI[u] = fetch(e_okI[u], e_offI[u], e_cl[u], c0, pa0, pb0);
      if (!diag) preJ[u] = fetch(e_okJ[u], e_offJ[u], e_cl[u], c0, pa0, pb0);
    }
  };
  // Operand addresses are invariant lane offsets plus constants: a wavefront takes its tiles one after
  // the other and, per tile, the 8 column pairs of the staged tile unrolled, so that nothing in the
  // loop but the matrix instructions needs the vector ALU (which they occupy).
  int offA[kGramMaxTiles], offB[kGramMaxTiles];       // doubles, from the start of a staged area
#pragma unroll
  for (int k = 0; k < kGramMaxTiles; ++k) {
    offA[k] = (16 * ti[k] + lrow) * kRowD + 4 * ccol + part;
    offB[k] = (16 * tj[k] + lrow) * kRowD + 4 * ccol + part;
  }
  auto multiply = [&](const double* bI, const double* bJ) {
#pragma unroll
    for (int k = 0; k < kGramMaxTiles; ++k) {
      if (mine[k]) {
        const double* pa = bI + offA[k];
        const double* pb = bJ + offB[k];
#pragma unroll
        for (int s2 = 0; s2 < kTC / 2; ++s2) {        // column 2 s2 + ccol: 4 doubles per column
          const double aRe = pa[8 * s2];              // part ? xi : xr
          const double aIm = pa[8 * s2 + 2];          // part ? -xr : xi
          const double bop = pb[8 * s2];
          accRe[k] = __builtin_amdgcn_mfma_f64_16x16x4f64(aRe, bop, accRe[k], 0, 0, 0);
          accIm[k] = __builtin_amdgcn_mfma_f64_16x16x4f64(aIm, bop, accIm[k], 0, 0, 0);
        }
      }
    }
  };
  if (diag) {
    // One staged side only, so the two LDS areas take turns: while the wavefronts multiply tile t out
    // of one, tile t + 1 is committed into the other (it was read last for tile t - 1, before the
    // barrier that ended that tile) and tile t + 2 is fetched into registers.  One barrier per tile.
    commit(sI, sI);
    if (c_begin + kTC < c_end) prefetch(c_begin + kTC);
    __syncthreads();
    int it = 0;
    for (int64_t c0 = c_begin; c0 < c_end; c0 += kTC, ++it) {
      double* cur = (it & 1) ? sJ : sI;
      double* nxt = (it & 1) ? sI : sJ;
      if (c0 + kTC < c_end) commit(nxt, nxt);
      if (c0 + 2 * kTC < c_end) prefetch(c0 + 2 * kTC);
      multiply(cur, cur);
      __syncthreads();
    }
  } else {
    for (int64_t c0 = c_begin; c0 < c_end; c0 += kTC) {
      __syncthreads();                                // previous tile fully consumed
      commit(sI, sJ);
      __syncthreads();
      if (c0 + kTC < c_end) prefetch(c0 + kTC);       // next 16 columns go in flight
      multiply(sI, sJ);
    }
  }
  double2* out = reinterpret_cast<double2*>(partials) + (int64_t)blockIdx.x * In * In;
#pragma unroll
  for (int k = 0; k < kGramMaxTiles; ++k) {
    if (mine[k]) {
      for (int r = 0; r < 4; ++r) {
        const int i = si * kSuper + 16 * ti[k] + 4 * r + (lane >> 4);
        const int j = sj * kSuper + 16 * tj[k] + (lane & 15);
        if (i < In && j < In) out[(int64_t)i * In + j] = make_double2(accRe[k][r], accIm[k][r]);
      }
    }
  }
}

// -------------------------------------------------------------------------------------------------
// k_gram128: the same Gram for extents In <= 128 - one super block, on the diagonal - which is every
// mode of the FNO shapes.  Same staging scheme and the same arithmetic as k_gram's diagonal case (the
// two LDS areas take turns, one barrier per staged tile of 16 columns); what differs is what runs
// next to the f64 matrix instructions, which occupy the SIMD's vector ALU as well:
//  * 8 wavefronts instead of 16 (256 registers each): the accumulators of 6 tiles and a fetched tile
//    stay in registers with nothing spilled.  (A spill reload is a vector-memory load: it waits for
//    every prefetch in flight and puts the memory latency back in front of the matrix phase.)
//  * Fetch: the element and its support-mask word come through two buffer descriptors (the tile's
//    first column as base, rebuilt in scalar registers per tile).  A lane's offset is invariant -
//    row * B + column, plus the wrap into the next leading index - and lanes without an element
//    (row >= In, column past the chunk) use an offset that the hardware range check answers with
//    zero: no branches, no 64-bit vector arithmetic.  The mask is applied when the tile is
//    committed to LDS, so nothing waits for the loads before the matrix phase.
//  * Matrix phase: a wavefront's tiles are runs inside one tile ROW, so the row-side operands
//    (xr | xi) and (xi | -xr) are fetched from LDS once per run and column pair (62 operand fetches
//    per column pair instead of 108), three column pairs ahead of the matrix instructions that use
//    them; the main loop exists once per shape of tile set, chosen outside the loop, so inside it
//    the accumulators live in fixed registers.
// With fewer than 8 tile rows (In <= 112) the tiles are dealt one by one as in k_gram.
struct GramRuns {                    // a wavefront's tiles when all 8 tile rows exist: run A = (ra, a0 .. a0 + na - 1),
  signed char ra, a0, na, rb, b0, nb;  // run B = (rb, b0 .. b0 + nb - 1), every run inside one tile row
};
// 36 tiles of the lower triangle over 8 wavefronts: 5 tiles for wavefronts 0..3, 4 tiles for 4..7
// (wavefronts w and w + 4 share a SIMD: 9 tiles per SIMD).  Wavefronts 5..7 hold one run of 4.
__constant__ GramRuns kGramRuns[8] = {
    {2, 0, 3, 1, 0, 2}, {4, 0, 3, 3, 0, 2}, {5, 0, 3, 3, 2, 2}, {5, 3, 3, 4, 3, 2},
    {6, 0, 3, 0, 0, 1}, {6, 3, 2, 6, 5, 2}, {7, 0, 2, 7, 2, 2}, {7, 4, 2, 7, 6, 2}};

constexpr int kGram128Threads = 512;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t gram_buffer(const void* base, uint32_t bytes) {
  // untyped buffer, stride 0: a load at an offset >= bytes returns zero
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), (short)0, (int)bytes, 0x00020000);
}

template <int DT, bool SMALLB>
__global__ __launch_bounds__(kGram128Threads) void k_gram128(const void* __restrict__ x,
                                                             const uint32_t* __restrict__ mask, int64_t A, int In,
                                                             int64_t B64, int64_t cols_per_chunk, uint32_t magicB,
                                                             double* __restrict__ partials) {
  extern __shared__ double sG[];
  constexpr int kEs = DT == TGRAD_C64 ? 8 : 4;        // bytes per element
  constexpr uint32_t kNowhere = 0xFFFFFFF0u;          // an offset beyond every descriptor: the load returns zero
  double* buf0 = sG;
  double* buf1 = sG + kSuper * kRowD;
  const uint32_t B = (uint32_t)B64;                   // the host takes this kernel only when In * B < 2^28
  const int64_t J = A * B64;
  const int64_t c_begin = (int64_t)blockIdx.x * cols_per_chunk;
  const int64_t c_end = c_begin + cols_per_chunk < J ? c_begin + cols_per_chunk : J;
  const bool empty = c_begin >= c_end;                // (workgroup-uniform) a trailing chunk without columns writes zeros
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int part = (lane >> 4) & 1, ccol = lane >> 5, lrow = lane & 15;
  const int ntr = (In + 15) >> 4;                     // tile rows present

  // ---- staging: a thread owns kPer elements (il, cl) of every staged tile ----
  constexpr int kPer = kSuper * kTC / kGram128Threads;   // 4
  // lane-invariant offset (elements) of (il, cl) from the tile's first column, before any wrap of the
  // column into the next leading index; rows that do not exist point nowhere
  const uint32_t wrap_add = (uint32_t)(In - 1) * B;
  uint32_t off0[kPer];
  int cl[kPer], lds_slot[kPer];
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int e = tid + u * kGram128Threads;
    int il;
    if (B == 1) { il = e % kSuper; cl[u] = e / kSuper; } else { il = e / kTC; cl[u] = e % kTC; }
    off0[u] = il < In ? (uint32_t)il * B + (uint32_t)cl[u] : kNowhere;
    lds_slot[u] = il * kRowD + 4 * cl[u];
  }
  const uint64_t total_bytes = (uint64_t)J * (uint64_t)In * kEs;
  const __amdgpu_buffer_rsrc_t rmask = gram_buffer(mask, mask ? (uint32_t)((((uint64_t)J * In + 31) >> 5) * 4) : 0u);

  // the tile being fetched: first column c = (a0, b0) (workgroup-uniform, scalar registers)
  uint32_t pa0 = (uint32_t)(c_begin / B64), pb0 = (uint32_t)(c_begin - (int64_t)pa0 * B64);
  uint32_t pre0[kPer], pre1[kPer];                    // the fetched elements as they lie in memory
  uint32_t pre_m[kPer], pre_g[kPer];                  // their mask words and global element indices
  auto fetch_tile = [&](int64_t c0) {                 // the tile that starts at column c0 = (pa0, pb0) -> pre
    const uint64_t base_e = (uint64_t)pa0 * (uint64_t)In * B + pb0;          // < 2^31 elements
    const uint64_t base_b = base_e * kEs;
    const uint64_t left = total_bytes - base_b;       // bytes of the tensor from the tile's first element on
    const __amdgpu_buffer_rsrc_t rx =
        gram_buffer(reinterpret_cast<const char*>(x) + base_b, left > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)left);
    const uint32_t lim = (uint32_t)(c_end - c0 < kTC ? c_end - c0 : kTC);    // columns of this tile inside the chunk
    const uint32_t base32 = (uint32_t)base_e;
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      uint32_t off;
      if constexpr (SMALLB) {                         // B < 16: (b0 + cl) / B wraps, b0 + cl < 32
        const uint32_t n = pb0 + (uint32_t)cl[u];
        const uint32_t q = magicB ? __umulhi(n, magicB) : n;
        off = off0[u] + q * wrap_add;
      } else {                                        // B >= 16: at most one wrap
        off = off0[u] + ((pb0 + (uint32_t)cl[u] >= B) ? wrap_add : 0u);
      }
      if (off0[u] == kNowhere || (uint32_t)cl[u] >= lim) off = kNowhere;
      const uint32_t gi = base32 + off;               // global element index (unused where off points nowhere)
      pre_g[u] = gi;
      const uint32_t voff = off == kNowhere ? kNowhere : off * kEs;
      if constexpr (DT == TGRAD_C64) {
        typedef uint32_t u2 __attribute__((ext_vector_type(2)));
        const u2 r = __builtin_amdgcn_raw_buffer_load_b64(rx, voff, 0, 0);
        pre0[u] = r.x;
        pre1[u] = r.y;
      } else {
        pre0[u] = __builtin_amdgcn_raw_buffer_load_b32(rx, voff, 0, 0);
        pre1[u] = 0u;
      }
      pre_m[u] = __builtin_amdgcn_raw_buffer_load_b32(rmask, off == kNowhere ? kNowhere : ((gi >> 5) << 2), 0, 0);
    }
  };
  auto next_tile = [&]() {
    pb0 += kTC;
    if constexpr (SMALLB) {
      const uint32_t q = magicB ? __umulhi(pb0, magicB) : pb0;
      pa0 += q;
      pb0 -= q * B;
    } else {
      if (pb0 >= B) { pb0 -= B; pa0 += 1; }
    }
  };
  auto commit = [&](double* d) {                      // pre -> one staged tile, as (xr, xi, xi, -xr) per element
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      float fr, fi;
      if constexpr (DT == TGRAD_C64) {
        fr = __uint_as_float(pre0[u]);
        fi = __uint_as_float(pre1[u]);
      } else {                                        // a bf16 is the upper half of a float32
        fr = __uint_as_float(pre0[u] << 16);
        fi = __uint_as_float(pre0[u] & 0xFFFF0000u);
      }
      const bool masked = (pre_m[u] >> (pre_g[u] & 31u)) & 1u;
      const double xr = (double)(masked ? 0.f : fr), xi = (double)(masked ? 0.f : fi);
      double2* q = reinterpret_cast<double2*>(d + lds_slot[u]);
      q[0] = make_double2(xr, xi);
      q[1] = make_double2(xi, -xr);
    }
  };

  // ---- this wavefront's tiles ----
  constexpr int kMaxT = 6;
  int ti[kMaxT], tj[kMaxT];
  bool mine[kMaxT];
  if (ntr == 8) {
    const GramRuns g = kGramRuns[wave];
#pragma unroll
    for (int k = 0; k < kMaxT; ++k) {
      const bool in_a = k < g.na;
      mine[k] = k < g.na + g.nb;
      ti[k] = in_a ? g.ra : g.rb;
      tj[k] = !mine[k] ? 0 : in_a ? g.a0 + k : g.b0 + (k - g.na);
    }
  } else {                                            // fewer tile rows: tile t of the lower triangle to wavefront t % 8
    const int ntl = ntr * (ntr + 1) / 2;
#pragma unroll
    for (int k = 0; k < kMaxT; ++k) {
      const int t = wave + 8 * k;
      int a = (int)((sqrtf(8.f * (float)t + 1.f) - 1.f) * 0.5f);
      while (a * (a + 1) / 2 > t) --a;
      while ((a + 1) * (a + 2) / 2 <= t) ++a;
      mine[k] = t < ntl;
      ti[k] = mine[k] ? a : 0;
      tj[k] = mine[k] ? t - a * (a + 1) / 2 : 0;
    }
  }
  v4d accRe[kMaxT], accIm[kMaxT];
#pragma unroll
  for (int k = 0; k < kMaxT; ++k) {
    accRe[k] = (v4d){0., 0., 0., 0.};
    accIm[k] = (v4d){0., 0., 0., 0.};
  }
  const int lane_off = lrow * kRowD + 4 * ccol + part;   // doubles, within a tile row of a staged area
  // A run of NT tiles of one tile row in accumulator slots S0 ..: the row-side operands are fetched
  // once per column pair for the whole run, kAhead - 1 column pairs ahead of the matrix instructions
  // (an LDS fetch right in front of its use leaves the matrix core idle for the LDS latency whenever
  // the SIMD's other wavefront is not ready).
  constexpr int kAhead = 3;
  auto multiply_run = [&](const double* b, auto s0_c, auto nt_c) {
    constexpr int S0 = decltype(s0_c)::value;
    constexpr int NT = decltype(nt_c)::value;
    const double* pa = b + 16 * ti[S0] * kRowD + lane_off;
    const double* pb[NT];
#pragma unroll
    for (int k = 0; k < NT; ++k) pb[k] = b + 16 * tj[S0 + k] * kRowD + lane_off;
    double ar[kAhead], ai[kAhead], bo[kAhead][NT];
    auto fetch_ops = [&](int s2) {                    // column 2 s2 + ccol: 4 doubles per column
      const int slot = s2 % kAhead;
      ar[slot] = pa[8 * s2];                          // part ? xi : xr
      ai[slot] = pa[8 * s2 + 2];                      // part ? -xr : xi
#pragma unroll
      for (int k = 0; k < NT; ++k) bo[slot][k] = pb[k][8 * s2];
    };
#pragma unroll
    for (int s2 = 0; s2 < kAhead - 1; ++s2) fetch_ops(s2);
#pragma unroll
    for (int s2 = 0; s2 < kTC / 2; ++s2) {
      if (s2 + kAhead - 1 < kTC / 2) fetch_ops(s2 + kAhead - 1);
      __builtin_amdgcn_sched_barrier(0);
      const int slot = s2 % kAhead;
#pragma unroll
      for (int k = 0; k < NT; ++k) {
        accRe[S0 + k] = __builtin_amdgcn_mfma_f64_16x16x4f64(ar[slot], bo[slot][k], accRe[S0 + k], 0, 0, 0);
        accIm[S0 + k] = __builtin_amdgcn_mfma_f64_16x16x4f64(ai[slot], bo[slot][k], accIm[S0 + k], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto multiply_single = [&](const double* b) {       // fewer than 8 tile rows: tile by tile
#pragma unroll
    for (int k = 0; k < kMaxT; ++k) {
      if (mine[k]) {
        const double* pa = b + 16 * ti[k] * kRowD + lane_off;
        const double* pb = b + 16 * tj[k] * kRowD + lane_off;
#pragma unroll
        for (int s2 = 0; s2 < kTC / 2; ++s2) {
          const double aRe = pa[8 * s2];
          const double aIm = pa[8 * s2 + 2];
          const double bop = pb[8 * s2];
          accRe[k] = __builtin_amdgcn_mfma_f64_16x16x4f64(aRe, bop, accRe[k], 0, 0, 0);
          accIm[k] = __builtin_amdgcn_mfma_f64_16x16x4f64(aIm, bop, accIm[k], 0, 0, 0);
        }
      }
    }
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  using I4 = std::integral_constant<int, 4>;

  // ---- main loop: while the wavefronts multiply tile t out of one LDS area, tile t + 1 is committed
  // into the other (read last for tile t - 1, before the barrier that ended it) and tile t + 2 is
  // fetched.  One instance of the loop per shape of a wavefront's tile set; every instance passes the
  // same barriers. ----
  auto main_loop = [&](auto na_c, auto nb_c) {        // (NA, NB): runs of NA and NB tiles; (0, 0): tile by tile
    constexpr int NA = decltype(na_c)::value;
    constexpr int NB = decltype(nb_c)::value;
    fetch_tile(c_begin);
    commit(buf0);
    if (c_begin + kTC < c_end) { next_tile(); fetch_tile(c_begin + kTC); }
    __syncthreads();
    int it = 0;
    for (int64_t c0 = c_begin; c0 < c_end; c0 += kTC, ++it) {
      double* cur = (it & 1) ? buf1 : buf0;
      double* nxt = (it & 1) ? buf0 : buf1;
      if (c0 + kTC < c_end) commit(nxt);
      if (c0 + 2 * kTC < c_end) { next_tile(); fetch_tile(c0 + 2 * kTC); }
      if constexpr (NA == 0) {
        multiply_single(cur);
      } else {
        multiply_run(cur, I0{}, na_c);
        if constexpr (NB > 0) multiply_run(cur, na_c, nb_c);
      }
      __syncthreads();
    }
  };
  if (!empty) {
    if (ntr != 8) main_loop(I0{}, I0{});
    else if (wave < 4) main_loop(I3{}, I2{});
    else if (wave == 4) main_loop(I3{}, I1{});
    else main_loop(I4{}, I0{});                        // both runs lie in one tile row: a run of 4
  }
  double2* out = reinterpret_cast<double2*>(partials) + (int64_t)blockIdx.x * In * In;
#pragma unroll
  for (int k = 0; k < kMaxT; ++k) {
    if (mine[k]) {
      for (int r = 0; r < 4; ++r) {
        const int i = 16 * ti[k] + 4 * r + (lane >> 4);
        const int j = 16 * tj[k] + (lane & 15);
        if (i < In && j < In) out[(int64_t)i * In + j] = make_double2(accRe[k][r], accIm[k][r]);
      }
    }
  }
}

// gram[i, j] = sum over chunks of partials[chunk][i, j] for i >= j; the upper triangle is the
// conjugate mirror (the Gram kernels leave it unwritten).  The chunks of one entry are summed by 8
// threads, each over a contiguous eighth of the chunks in order, and the 8 partial sums are added in
// order: the result does not depend on the launch, and 8 times as many loads are in flight.
constexpr int kReduceSplit = 8;
constexpr int kReduceElems = 256 / kReduceSplit;     // entries per workgroup
__global__ __launch_bounds__(256) void k_gram_reduce(const double* __restrict__ partials, int nchunks, int In,
                                                     double* __restrict__ gram) {
  __shared__ double2 part[kReduceSplit][kReduceElems];
  const int el = threadIdx.x % kReduceElems, sub = threadIdx.x / kReduceElems;
  const int64_t e = (int64_t)blockIdx.x * kReduceElems + el;
  const int64_t n2 = (int64_t)In * In;
  const bool in = e < n2;
  const int i = in ? (int)(e / In) : 0, j = in ? (int)(e - (int64_t)i * In) : 0;
  const int64_t src = i >= j ? (int64_t)i * In + j : (int64_t)j * In + i;
  const int per = (nchunks + kReduceSplit - 1) / kReduceSplit;
  const int c0 = sub * per, c1 = c0 + per < nchunks ? c0 + per : nchunks;
  const double2* p2 = reinterpret_cast<const double2*>(partials);
  double re = 0., im = 0.;
  if (in)
    for (int c = c0; c < c1; ++c) {
      const double2 v = p2[(int64_t)c * n2 + src];
      re += v.x;
      im += v.y;
    }
  part[sub][el] = make_double2(re, im);
  __syncthreads();
  if (sub == 0 && in) {
    double sr = 0., si = 0.;
#pragma unroll
    for (int q = 0; q < kReduceSplit; ++q) {
      sr += part[q][el].x;
      si += part[q][el].y;
    }
    reinterpret_cast<double2*>(gram)[e] = make_double2(sr, i >= j ? si : -si);
  }
}

// ---------------------------------------------------------------------------------------------
// Hermitian eigen-solve by parallel cyclic Jacobi (two-sided rotations, round-robin pairing).
// One workgroup per matrix; A and V live in global memory (L2-resident, <= 1 MiB each).
struct EigJob {
  const double* gram;   // n x n complex (interleaved), row-major
  double* A;            // work copy
  double* V;            // eigenvector accumulator
  float* U;             // out: n x r complex float32, row-major
  int* status;          // out: [0] = 1 if the solve stopped at the sweep limit with rotations left, else 0;
                        //      [1] = Jacobi sweeps run; [2] = 1 if the tridiagonal path declined (close eigenvalues)
  int n;
  int r;
  int max_sweeps;
  int use_fast;         // 1: Householder tridiagonalisation + bisection + inverse iteration first (n <= 128), the
                        //    Jacobi kernels run only if that path declines (status[2] != 0); 0: Jacobi
};
struct EigJobs {
  EigJob job[kMaxNdim];
};

// Rotation log of the LDS solver (extents <= 128), kept in the job's work buffer `A`: a header,
// then one entry per (logged round, slot).  p < 0: the slot's pivot was already negligible.
struct RotLog {
  double c, sx, sy;     // cos, sin e^{i phi}
  int p, q;
};
struct EigLogHeader {
  double lam[128];      // eigenvalues (diagonal of the converged work matrix)
  int rounds;           // logged rounds (rounds in which nothing rotates are not logged)
  int pad[3];
};

constexpr int kEigThreads = 1024;
constexpr int kEigMaxN = TGRAD_MAX_EXTENT;
constexpr int kEigMaxSweeps = 30;
constexpr int kEigBatch = 4;           // rotations per thread whose loads are in flight together

__device__ __forceinline__ double2 cmuld(double2 a, double2 b) {
  return make_double2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ double2 conjd(double2 a) { return make_double2(a.x, -a.y); }

// Shared tail of the eigensolvers: order the eigenvalues in `lam` descending (ties: lower index
// first), keep the first r, give every kept column of V the unit phase that makes its
// largest-modulus entry (first on ties) real and positive, and write U (n x r, float32).
__device__ void eig_finish(int n, int r, int tid, const double* lam, int* col_of, double2* phase,
                           const double2* V, float2* U) {
  for (int i = tid; i < n; i += kEigThreads) {
    int rank = 0;
    const double li = lam[i];
    for (int j = 0; j < n; ++j) rank += (lam[j] > li || (lam[j] == li && j < i)) ? 1 : 0;
    if (rank < r) col_of[rank] = i;
  }
  __syncthreads();
  for (int cidx = tid; cidx < r; cidx += kEigThreads) {
    const int src = col_of[cidx];
    double best = -1.;
    double2 vb = make_double2(1., 0.);
    for (int i = 0; i < n; ++i) {
      const double2 v = V[i * n + src];
      const double a2 = v.x * v.x + v.y * v.y;
      if (a2 > best) {
        best = a2;
        vb = v;
      }
    }
    const double mag = sqrt(best);
    phase[cidx] = mag > 0. ? make_double2(vb.x / mag, -vb.y / mag) : make_double2(1., 0.);
  }
  __syncthreads();
  for (int e = tid; e < n * r; e += kEigThreads) {
    const int i = e / r, cidx = e - i * r;
    const double2 v = cmuld(V[i * n + col_of[cidx]], phase[cidx]);
    U[e] = make_float2((float)v.x, (float)v.y);
  }
}

// Pair (p, q), p < q, of round `round` for slot `slot` of the round-robin tournament on m players.
__device__ __forceinline__ void jacobi_pair(int slot, int round, int m, int& p, int& q) {
  if (slot == 0) {
    p = m - 1;
    q = round;
  } else {
    p = (round + slot) % (m - 1);
    q = (round - slot + (m - 1)) % (m - 1);
  }
  if (p > q) {
    const int t = p;
    p = q;
    q = t;
  }
}

// Rotation that annihilates a_pq of the Hermitian 2 x 2 pivot [[app, apq], [conj(apq), aqq]]:
// c = cos, s = sin e^{i phi}.  Returns false (c = 1, s = 0) when a_pq is already negligible.
__device__ __forceinline__ bool jacobi_rotation(double app, double aqq, double2 apq, double eps2, double floor2,
                                                double& c, double2& s) {
  c = 1.;
  s = make_double2(0., 0.);
  const double mag2 = apq.x * apq.x + apq.y * apq.y;
  if (!(mag2 > eps2 * fabs(app * aqq) && mag2 > floor2)) return false;
  // two reciprocal square roots, one square root and one division (the threads that compute the
  // rotations are the critical path of a round: every other wavefront waits for them)
  const double inv_mag = rsqrt(mag2);
  const double tau = 0.5 * (aqq - app) * inv_mag;
  const double t = (tau >= 0. ? 1. : -1.) / (fabs(tau) + sqrt(1. + tau * tau));
  c = rsqrt(1. + t * t);
  const double sn = t * c * inv_mag;
  s = make_double2(sn * apq.x, sn * apq.y);
  return true;
}

__global__ __launch_bounds__(kEigThreads) void k_eig(EigJobs jobs) {
  const EigJob jb = jobs.job[blockIdx.x];
  const int n = jb.n, r = jb.r;
  const int tid = threadIdx.x;
  double2* A = reinterpret_cast<double2*>(jb.A);
  double2* V = reinterpret_cast<double2*>(jb.V);
  const double2* G = reinterpret_cast<const double2*>(jb.gram);

  __shared__ int sp[kEigMaxN / 2 + 1], sq[kEigMaxN / 2 + 1];
  __shared__ double sc[kEigMaxN / 2 + 1];       // cos
  __shared__ double2 ss[kEigMaxN / 2 + 1];      // sin * e^{i phi}
  __shared__ int srot[kEigMaxN / 2 + 1];        // 1 if this pair rotates in this round
  __shared__ int nrot;
  __shared__ double red[kEigThreads];
  __shared__ double lam[kEigMaxN];
  __shared__ int col_of[kEigMaxN];
  __shared__ double2 phase[kEigMaxN];

  // A <- gram, V <- I, trace
  double tr = 0.;
  for (int e = tid; e < n * n; e += kEigThreads) {
    double2 g = G[e];
    A[e] = g;
    const int i = e / n, j = e - i * n;
    V[e] = make_double2(i == j ? 1. : 0., 0.);
    if (i == j) tr += g.x;
  }
  red[tid] = tr;
  __syncthreads();
  for (int off = kEigThreads / 2; off > 0; off >>= 1) {
    if (tid < off) red[tid] += red[tid + off];
    __syncthreads();
  }
  const double trace = red[0];
  const double floor2 = (2.2e-18 * trace / n) * (2.2e-18 * trace / n);   // (1e-2 eps mean-eigenvalue)^2
  const double eps2 = 4.93e-32;                                          // (2^-52)^2
  const int m = n + (n & 1);                                             // even player count
  const int half = m / 2;

  int sweeps_run = 0, converged = 0;
  for (int sweep = 0; sweep < jb.max_sweeps; ++sweep) {
    if (tid == 0) nrot = 0;
    __syncthreads();
    for (int round = 0; round < m - 1; ++round) {
      // ---- phase 1: pairs of this round and their rotations ----
      if (tid < half) {
        int p, q;
        jacobi_pair(tid, round, m, p, q);
        int rot = 0;
        double c = 1.;
        double2 s = make_double2(0., 0.);
        if (q < n)                                     // q == n is the padding player of an odd n
          rot = jacobi_rotation(A[p * n + p].x, A[q * n + q].x, A[p * n + q], eps2, floor2, c, s) ? 1 : 0;
        sp[tid] = p;
        sq[tid] = q;
        sc[tid] = c;
        ss[tid] = s;
        srot[tid] = rot;
        if (rot) atomicAdd(&nrot, 1);
      }
      __syncthreads();
      // ---- phase 2: column rotations  X[:, p] <- c X[:, p] - conj(s) X[:, q],
      //                                 X[:, q] <- s X[:, p] + c X[:, q]   for X in {A, V} ----
      // (loads of a batch are all issued before the first use: one memory round trip per batch)
      for (int e0 = tid; e0 < 2 * n * half; e0 += kEigThreads * kEigBatch) {
        double2 xp[kEigBatch], xq[kEigBatch];
        int off_p[kEigBatch], off_q[kEigBatch], prs[kEigBatch];      // prs: pair | (matrix << 16), -1 = idle
#pragma unroll
        for (int u = 0; u < kEigBatch; ++u) {
          const int e = e0 + u * kEigThreads;
          prs[u] = -1;
          if (e < 2 * n * half) {
            const int which = e / (n * half);
            const int e2 = e - which * (n * half);
            const int i = e2 / half, pr = e2 - i * half;
            if (srot[pr]) {
              const double2* X = which ? V : A;
              prs[u] = pr | (which << 16);
              off_p[u] = i * n + sp[pr];
              off_q[u] = i * n + sq[pr];
              xp[u] = X[off_p[u]];
              xq[u] = X[off_q[u]];
            }
          }
        }
#pragma unroll
        for (int u = 0; u < kEigBatch; ++u) {
          if (prs[u] >= 0) {
            double2* X = (prs[u] >> 16) ? V : A;
            const int pr = prs[u] & 0xFFFF;
            const double c = sc[pr];
            const double2 s = ss[pr];
            const double2 t1 = cmuld(conjd(s), xq[u]), t2 = cmuld(s, xp[u]);
            X[off_p[u]] = make_double2(c * xp[u].x - t1.x, c * xp[u].y - t1.y);
            X[off_q[u]] = make_double2(t2.x + c * xq[u].x, t2.y + c * xq[u].y);
          }
        }
      }
      __syncthreads();
      // ---- phase 3: row rotations  A[p, :] <- c A[p, :] - s A[q, :],
      //                              A[q, :] <- conj(s) A[p, :] + c A[q, :] ----
      for (int e0 = tid; e0 < half * n; e0 += kEigThreads * kEigBatch) {
        double2 xp[kEigBatch], xq[kEigBatch];
        int off_p[kEigBatch], off_q[kEigBatch], prs[kEigBatch];
#pragma unroll
        for (int u = 0; u < kEigBatch; ++u) {
          const int e = e0 + u * kEigThreads;
          prs[u] = -1;
          if (e < half * n) {
            const int pr = e / n, j = e - pr * n;
            if (srot[pr]) {
              prs[u] = pr;
              off_p[u] = sp[pr] * n + j;
              off_q[u] = sq[pr] * n + j;
              xp[u] = A[off_p[u]];
              xq[u] = A[off_q[u]];
            }
          }
        }
#pragma unroll
        for (int u = 0; u < kEigBatch; ++u) {
          if (prs[u] >= 0) {
            const double c = sc[prs[u]];
            const double2 s = ss[prs[u]];
            const double2 t1 = cmuld(s, xq[u]), t2 = cmuld(conjd(s), xp[u]);
            A[off_p[u]] = make_double2(c * xp[u].x - t1.x, c * xp[u].y - t1.y);
            A[off_q[u]] = make_double2(t2.x + c * xq[u].x, t2.y + c * xq[u].y);
          }
        }
      }
      __syncthreads();
    }
    const int done = (nrot == 0);
    __syncthreads();
    ++sweeps_run;
    if (done) {
      converged = 1;
      break;
    }
  }
  if (tid == 0) {
    jb.status[0] = converged ? 0 : 1;
    jb.status[1] = sweeps_run;
  }

  for (int i = tid; i < n; i += kEigThreads) lam[i] = A[i * n + i].x;
  __syncthreads();
  eig_finish(n, r, tid, lam, col_of, phase, V, reinterpret_cast<float2*>(jb.U));
}

// The same solver for n <= 128 with the Hermitian work matrix held in LDS (lower triangle,
// n (n + 1) / 2 complex doubles <= 132 KB): a round is then one barrier-separated pair of phases
// on LDS - rotations from the pivots, then every 2 x 2 block (pair a, pair b), a >= b, updated in one
// step as  L_a B R_b  (the column and the row rotation of the two-pass form fused) - and only the
// eigenvector accumulator V goes through memory, once per round.
constexpr int kEigTriMaxN = 128;

__device__ __forceinline__ int tri_idx(int i, int j) { return i * (i + 1) / 2 + j; }           // i >= j
__device__ __forceinline__ double2 tri_get(const double2* T, int i, int j) {
  return i >= j ? T[tri_idx(i, j)] : conjd(T[tri_idx(j, i)]);
}
__device__ __forceinline__ void tri_put(double2* T, int i, int j, double2 v) {
  if (i >= j) T[tri_idx(i, j)] = v; else T[tri_idx(j, i)] = conjd(v);
}

__global__ __launch_bounds__(kEigThreads) void k_eig_tri(EigJobs jobs) {
  extern __shared__ double2 T[];                // lower triangle of the work matrix
  const EigJob jb = jobs.job[blockIdx.x];
  if (jb.use_fast && jb.status[2] == 0) return;   // the tridiagonal path has delivered this factor
  const int n = jb.n;
  const int tid = threadIdx.x;
  const double2* G = reinterpret_cast<const double2*>(jb.gram);
  EigLogHeader* hdr = reinterpret_cast<EigLogHeader*>(jb.A);
  RotLog* rlog = reinterpret_cast<RotLog*>(reinterpret_cast<char*>(jb.A) + sizeof(EigLogHeader));
  int nlogged = 0;                               // rounds written to the log (uniform over the block)

  __shared__ int sp[kEigTriMaxN / 2 + 1], sq[kEigTriMaxN / 2 + 1];
  __shared__ double sc[kEigTriMaxN / 2 + 1];
  __shared__ double2 ss[kEigTriMaxN / 2 + 1];
  __shared__ int srot[kEigTriMaxN / 2 + 1];
  __shared__ int nrot;
  __shared__ double red[kEigThreads];

  double tr = 0.;
  for (int e = tid; e < n * n; e += kEigThreads) {
    const int i = e / n, j = e - i * n;
    const double2 g = G[e];
    if (i >= j) T[tri_idx(i, j)] = g;
    if (i == j) tr += g.x;
  }
  red[tid] = tr;
  __syncthreads();
  for (int off = kEigThreads / 2; off > 0; off >>= 1) {
    if (tid < off) red[tid] += red[tid + off];
    __syncthreads();
  }
  const double trace = red[0];
  const double floor2 = (2.2e-18 * trace / n) * (2.2e-18 * trace / n);
  const double eps2 = 4.93e-32;
  const int m = n + (n & 1);
  const int half = m / 2;
  const int nblocks = half * (half - 1) / 2;
  // The off-pivot blocks (pair a, pair b), a > b, a thread updates in every round: e = tid, tid + 1024
  // (2016 blocks for 64 pairs: two per thread); decoded once, packed as a << 8 | b, -1 = none.  The
  // pivot block (a, a) is updated by the thread that computes its rotation.
  constexpr int kBlocksPerThread = (kEigTriMaxN / 2) * (kEigTriMaxN / 2 - 1) / 2 / kEigThreads + 1;
  int my_ab[kBlocksPerThread];
#pragma unroll
  for (int u = 0; u < kBlocksPerThread; ++u) {
    const int e = tid + u * kEigThreads;
    my_ab[u] = -1;
    if (e < nblocks) {
      int a = (int)((sqrtf(8.f * (float)e + 1.f) + 1.f) * 0.5f);
      while (a * (a - 1) / 2 > e) --a;
      while ((a + 1) * a / 2 <= e) ++a;
      my_ab[u] = (a << 8) | (e - a * (a - 1) / 2);
    }
  }
  // B <- L_a B R_b for the 2 x 2 block (rows p_a, q_a; columns p_b, q_b), L = [[c, -s], [conj(s), c]],
  // R = [[c, s], [-conj(s), c]]; a == b: the pivot block, of which the lower triangle is kept
  auto update_block = [&](int a, int b) {
    const int pa = sp[a], qa = sq[a], pb = sp[b], qb = sq[b];
    const bool qa_ok = qa < n, qb_ok = qb < n;         // padding player of an odd n: no such row / column
    const double ca = sc[a], cb = sc[b];
    const double2 sa = ss[a], sb = ss[b];
    const double2 zero = make_double2(0., 0.);
    double2 b00 = tri_get(T, pa, pb);
    double2 b01 = qb_ok ? tri_get(T, pa, qb) : zero;
    double2 b10 = qa_ok ? tri_get(T, qa, pb) : zero;
    double2 b11 = (qa_ok && qb_ok) ? tri_get(T, qa, qb) : zero;
    // rows: [r_p; r_q] <- [c r_p - s r_q; conj(s) r_p + c r_q]
    {
      const double2 t00 = cmuld(sa, b10), t01 = cmuld(sa, b11);
      const double2 u00 = cmuld(conjd(sa), b00), u01 = cmuld(conjd(sa), b01);
      const double2 n00 = make_double2(ca * b00.x - t00.x, ca * b00.y - t00.y);
      const double2 n01 = make_double2(ca * b01.x - t01.x, ca * b01.y - t01.y);
      const double2 n10 = make_double2(u00.x + ca * b10.x, u00.y + ca * b10.y);
      const double2 n11 = make_double2(u01.x + ca * b11.x, u01.y + ca * b11.y);
      b00 = n00; b01 = n01; b10 = n10; b11 = n11;
    }
    // columns: [x_p, x_q] <- [c x_p - conj(s) x_q, s x_p + c x_q]
    {
      const double2 t00 = cmuld(conjd(sb), b01), t10 = cmuld(conjd(sb), b11);
      const double2 u00 = cmuld(sb, b00), u10 = cmuld(sb, b10);
      const double2 n00 = make_double2(cb * b00.x - t00.x, cb * b00.y - t00.y);
      const double2 n10 = make_double2(cb * b10.x - t10.x, cb * b10.y - t10.y);
      const double2 n01 = make_double2(u00.x + cb * b01.x, u00.y + cb * b01.y);
      const double2 n11 = make_double2(u10.x + cb * b11.x, u10.y + cb * b11.y);
      b00 = n00; b01 = n01; b10 = n10; b11 = n11;
    }
    if (a == b) {
      T[tri_idx(pa, pa)] = b00;
      if (qa_ok) {
        T[tri_idx(qa, qa)] = b11;
        T[tri_idx(qa, pa)] = b10;
      }
    } else {
      tri_put(T, pa, pb, b00);
      if (qb_ok) tri_put(T, pa, qb, b01);
      if (qa_ok) tri_put(T, qa, pb, b10);
      if (qa_ok && qb_ok) tri_put(T, qa, qb, b11);
    }
  };

  int sweeps_run = 0, converged = 0;
  for (int sweep = 0; sweep < jb.max_sweeps; ++sweep) {
    if (tid == 0) nrot = 0;
    __syncthreads();
    for (int round = 0; round < m - 1; ++round) {
      // ---- phase 1: pairs of this round and their rotations ----
      int rot = 0;
      if (tid < half) {
        int p, q;
        jacobi_pair(tid, round, m, p, q);
        double c = 1.;
        double2 s = make_double2(0., 0.);
        if (q < n)                                     // a_pq = conj(T[q, p]) since p < q
          rot = jacobi_rotation(T[tri_idx(p, p)].x, T[tri_idx(q, q)].x, conjd(T[tri_idx(q, p)]), eps2, floor2,
                                c, s) ? 1 : 0;
        sp[tid] = p;
        sq[tid] = q;
        sc[tid] = c;
        ss[tid] = s;
        srot[tid] = rot;
        if (rot) atomicAdd(&nrot, 1);
      }
      if (!__syncthreads_or(rot)) continue;            // nothing rotates in this round (late sweeps)
      // ---- phase 2a: the round's rotations go to the log; the eigenvector accumulator is built from
      //      it afterwards by k_eig_apply, all rows in parallel ----
      if (tid < half) {
        RotLog e;
        e.c = sc[tid];
        e.sx = ss[tid].x;
        e.sy = ss[tid].y;
        e.p = srot[tid] ? sp[tid] : -1;
        e.q = sq[tid];
        rlog[(size_t)nlogged * half + tid] = e;
      }
      ++nlogged;
      // ---- phase 2b: every block (pair a, pair b), a >= b:  B <- L_a B R_b ----
      if (tid < half && srot[tid]) update_block(tid, tid);   // own pivot block (nobody else touches it)
#pragma unroll
      for (int u = 0; u < kBlocksPerThread; ++u) {
        if (my_ab[u] < 0) continue;
        const int a = my_ab[u] >> 8, b = my_ab[u] & 255;
        if (!srot[a] && !srot[b]) continue;
        update_block(a, b);
      }
      __syncthreads();
    }
    const int done = (nrot == 0);
    __syncthreads();
    ++sweeps_run;
    if (done) {
      converged = 1;
      break;
    }
  }
  for (int i = tid; i < n; i += kEigThreads) hdr->lam[i] = T[tri_idx(i, i)].x;
  if (tid == 0) {
    hdr->rounds = nlogged;
    jb.status[0] = converged ? 0 : 1;
    jb.status[1] = sweeps_run;
  }
}

// Eigenvector accumulator from the rotation log: V = R_1 R_2 ... (every round's rotations act on
// column pairs), so each ROW of V evolves on its own: one wavefront per row, the row in LDS, lane =
// slot of the round; the arithmetic per element is that of the in-kernel update of k_eig.
constexpr int kLogAhead = 4;                     // rounds whose log entries are in flight

__global__ __launch_bounds__(64) void k_eig_apply(EigJobs jobs) {
  const EigJob jb = jobs.job[blockIdx.y];
  if (jb.use_fast && jb.status[2] == 0) return;
  const int n = jb.n;
  const int row = blockIdx.x;
  if (row >= n) return;
  __shared__ double2 x[kEigTriMaxN];
  const int lane = threadIdx.x;
  for (int j = lane; j < n; j += 64) x[j] = make_double2(j == row ? 1. : 0., 0.);
  const EigLogHeader* hdr = reinterpret_cast<const EigLogHeader*>(jb.A);
  const RotLog* rlog = reinterpret_cast<const RotLog*>(reinterpret_cast<const char*>(jb.A) + sizeof(EigLogHeader));
  const int half = (n + (n & 1)) / 2;
  const int rounds = hdr->rounds;
  const int slot = lane < half ? lane : half - 1;          // idle lanes shadow the last slot, write nothing
  RotLog ahead[kLogAhead];
#pragma unroll
  for (int d = 0; d < kLogAhead; ++d) ahead[d] = rlog[(size_t)(d < rounds ? d : 0) * half + slot];
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  for (int r0 = 0; r0 < rounds; r0 += kLogAhead) {
#pragma unroll
    for (int d = 0; d < kLogAhead; ++d) {
      const int rr = r0 + d;
      const RotLog e = ahead[d];
      const int nxt = rr + kLogAhead;
      ahead[d] = rlog[(size_t)(nxt < rounds ? nxt : 0) * half + slot];
      if (rr < rounds && lane < half && e.p >= 0) {
        const double2 xp = x[e.p], xq = x[e.q];
        const double2 sc_ = make_double2(e.sx, e.sy);
        const double2 t1 = cmuld(conjd(sc_), xq), t2 = cmuld(sc_, xp);
        x[e.p] = make_double2(e.c * xp.x - t1.x, e.c * xp.y - t1.y);
        x[e.q] = make_double2(t2.x + e.c * xq.x, t2.y + e.c * xq.y);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the next round reads what this one wrote
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  }
  double2* V = reinterpret_cast<double2*>(jb.V);
  for (int j = lane; j < n; j += 64) V[(size_t)row * n + j] = x[j];
}

// Ordering, phase convention and the float32 factor, from the eigenvalues in the log header and V.
__global__ __launch_bounds__(kEigThreads) void k_eig_finish(EigJobs jobs) {
  const EigJob jb = jobs.job[blockIdx.x];
  if (jb.use_fast && jb.status[2] == 0) return;
  __shared__ double lam[kEigTriMaxN];
  __shared__ int col_of[kEigTriMaxN];
  __shared__ double2 phase[kEigTriMaxN];
  const EigLogHeader* hdr = reinterpret_cast<const EigLogHeader*>(jb.A);
  for (int i = threadIdx.x; i < jb.n; i += kEigThreads) lam[i] = hdr->lam[i];
  __syncthreads();
  eig_finish(jb.n, jb.r, threadIdx.x, lam, col_of, phase, reinterpret_cast<const double2*>(jb.V),
             reinterpret_cast<float2*>(jb.U));
}

// ---------------------------------------------------------------------------------------------
// The same eigenvectors by the classical three-stage route, for n <= 128 (one workgroup per matrix):
//   (1) Householder tridiagonalisation  A = Q T Q^H  of the Hermitian matrix (packed lower triangle
//       in LDS; reflector i annihilates column i below the subdiagonal; T real symmetric tridiagonal),
//   (2) the r largest eigenvalues of T by multisection on Sturm counts (32 lanes per eigenvalue, 32
//       points per step: 13 steps from the Gershgorin interval down to rounding),
//   (3) their eigenvectors by inverse iteration (Gaussian elimination with partial pivoting on
//       T - lambda I, three solves from a fixed pseudo-random start vector, one thread per vector),
//   (4) back-transformation with the reflectors, phase convention and the float32 factor (k_trid_back,
//       one wavefront per eigenvector).
// A cyclic Jacobi sweep reads and writes the whole matrix in every one of its n - 1 rounds, about
// ten sweeps long; the tridiagonalisation touches the trailing block once per step: 15 times less
// LDS traffic, which is what bounds both.
// Inverse iteration separates eigenvectors only as well as their eigenvalues are separated: if two
// of the r leading eigenvalues, or the r-th and the (r+1)-th, lie within 1e-7 of the spectral radius
// (exactly repeated eigenvalues, a zero matrix), this path declines (status[2] = 1) and the Jacobi
// kernels, which handle clusters gracefully, solve the matrix instead.
constexpr int kTridThreads = 1024;
constexpr int kInvBatch = 32;          // eigenvectors per inverse-iteration batch (LDS: 4 arrays of n x 32 doubles)
constexpr int kMultiSteps = 13;        // 33^13 > 2^64
constexpr double kClusterTol = 1e-7;

__device__ __forceinline__ double2* trid_tau(const EigJob& jb) { return reinterpret_cast<double2*>(jb.A); }
__device__ __forceinline__ double* trid_Z(const EigJob& jb) { return jb.A + 2 * jb.n; }   // r vectors of n doubles

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// 1 / q from the hardware's reciprocal estimate and two Newton steps (relative error a few 1e-16): the
// sequential recurrences below spend their time in this, and a correctly rounded float64 division
// is four times as long.  Their results only steer a bisection and an inverse iteration.
__device__ __forceinline__ double rcp_nr(double q) {
  double r = __builtin_amdgcn_rcp(q);
  r = fma(fma(-q, r, 1.), r, r);
  r = fma(fma(-q, r, 1.), r, r);
  return r;
}

// eigenvalues of the tridiagonal (d, e2 = e^2) below x
__device__ __forceinline__ int sturm_count(const double* d, const double* e2, int n, double x, double pivmin) {
  double q = d[0] - x;
  if (fabs(q) < pivmin) q = -pivmin;
  int c = q < 0. ? 1 : 0;
  for (int i = 1; i < n; ++i) {
    q = (d[i] - x) - e2[i - 1] * rcp_nr(q);
    if (fabs(q) < pivmin) q = -pivmin;
    c += q < 0. ? 1 : 0;
  }
  return c;
}

__device__ __forceinline__ uint32_t trid_mix(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  x *= 0x846CA68Bu;
  x ^= x >> 16;
  return x;
}

__global__ __launch_bounds__(kTridThreads) void k_trid(EigJobs jobs) {
  extern __shared__ double2 T[];                // packed lower triangle; reused by the inverse iteration
  const EigJob jb = jobs.job[blockIdx.x];
  const int n = jb.n, r = jb.r;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double2* G = reinterpret_cast<const double2*>(jb.gram);
  double2* Vg = reinterpret_cast<double2*>(jb.V);   // reflector i: Vg[i * n + row], rows i + 1 .. n - 1
  double2* tauG = trid_tau(jb);
  __shared__ double2 sv[kEigTriMaxN], sw[kEigTriMaxN];
  __shared__ double sd[kEigTriMaxN], se[kEigTriMaxN], se2[kEigTriMaxN], slam[kEigTriMaxN];
  __shared__ double2 s_tau, s_scale, s_alpha2;
  __shared__ double s_gl, s_gu, s_pivmin;
  __shared__ int s_decline;

  for (int e = tid; e < n * n; e += kTridThreads) {
    const int i = e / n, j = e - i * n;
    if (i >= j) T[tri_idx(i, j)] = G[e];
  }
  if (tid == 0) s_decline = 0;
  __syncthreads();

  // ---- (1) tridiagonalisation ----
  for (int i = 0; i + 1 < n; ++i) {
    const int m = n - i - 1;                     // trailing block: rows / columns i + 1 .. n - 1 (local 0 .. m - 1)
    if (wave == 0) {
      double xn2 = 0.;
      for (int j = 1 + lane; j < m; j += 64) {
        const double2 x = T[tri_idx(i + 1 + j, i)];
        xn2 += x.x * x.x + x.y * x.y;
      }
      xn2 = wave_sum_d(xn2);
      if (lane == 0) {
        const double2 alpha = T[tri_idx(i + 1, i)];
        double2 tau = make_double2(0., 0.), scale = make_double2(0., 0.);
        double beta = alpha.x;
        if (!(xn2 == 0. && alpha.y == 0.)) {
          beta = -copysign(sqrt(alpha.x * alpha.x + alpha.y * alpha.y + xn2), alpha.x);
          tau = make_double2((beta - alpha.x) / beta, -alpha.y / beta);
          const double2 z = make_double2(alpha.x - beta, alpha.y);          // 1 / (alpha - beta)
          const double inv = 1. / (z.x * z.x + z.y * z.y);
          scale = make_double2(z.x * inv, -z.y * inv);
        }
        s_tau = tau;
        s_scale = scale;
        se[i] = beta;
        sd[i] = T[tri_idx(i, i)].x;
        tauG[i] = tau;
      }
    }
    __syncthreads();
    const double2 tau = s_tau;
    const bool reflect = tau.x != 0. || tau.y != 0.;           // (workgroup-uniform)
    for (int j = tid; j < m; j += kTridThreads) {
      double2 v = make_double2(j == 0 ? 1. : 0., 0.);
      if (j > 0 && reflect) v = cmuld(T[tri_idx(i + 1 + j, i)], s_scale);
      sv[j] = v;
      Vg[(size_t)i * n + i + 1 + j] = v;
    }
    __syncthreads();
    if (!reflect) continue;
    // p = tau S v: 8 threads per row, each over the columns c = q, q + 8, ..; summed in a fixed order
    {
      const int rr = tid >> 3, q = tid & 7;
      double2 acc = make_double2(0., 0.);
      if (rr < m)
        for (int c = q; c < m; c += 8) {
          const double2 sv_c = sv[c];
          const double2 a = c <= rr ? T[tri_idx(i + 1 + rr, i + 1 + c)] : conjd(T[tri_idx(i + 1 + c, i + 1 + rr)]);
          const double2 t = cmuld(a, sv_c);
          acc.x += t.x;
          acc.y += t.y;
        }
#pragma unroll
      for (int off = 1; off < 8; off <<= 1) {
        acc.x += __shfl_xor(acc.x, off, 64);
        acc.y += __shfl_xor(acc.y, off, 64);
      }
      if (q == 0 && rr < m) sw[rr] = cmuld(tau, acc);
    }
    __syncthreads();
    // alpha2 = -1/2 tau (p^H v);  w = p + alpha2 v
    if (wave == 0) {
      double ax = 0., ay = 0.;
      for (int j = lane; j < m; j += 64) {
        const double2 t = cmuld(conjd(sw[j]), sv[j]);
        ax += t.x;
        ay += t.y;
      }
      ax = wave_sum_d(ax);
      ay = wave_sum_d(ay);
      if (lane == 0) {
        const double2 t = cmuld(tau, make_double2(ax, ay));
        s_alpha2 = make_double2(-0.5 * t.x, -0.5 * t.y);
      }
    }
    __syncthreads();
    for (int j = tid; j < m; j += kTridThreads) {
      const double2 t = cmuld(s_alpha2, sv[j]);
      sw[j] = make_double2(sw[j].x + t.x, sw[j].y + t.y);
    }
    __syncthreads();
    // S <- S - v w^H - w v^H on the lower triangle
    {
      const int ty = tid >> 5, tx = tid & 31;
      for (int rr = ty; rr < m; rr += 32) {
        const double2 vr = sv[rr], wr = sw[rr];
        for (int c = tx; c <= rr; c += 32) {
          const double2 t1 = cmuld(vr, conjd(sw[c])), t2 = cmuld(wr, conjd(sv[c]));
          double2* p = &T[tri_idx(i + 1 + rr, i + 1 + c)];
          *p = make_double2(p->x - t1.x - t2.x, p->y - t1.y - t2.y);
        }
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    sd[n - 1] = T[tri_idx(n - 1, n - 1)].x;
    se[n - 1] = 0.;
  }
  __syncthreads();
  for (int i = tid; i < n; i += kTridThreads) se2[i] = se[i] * se[i];
  __syncthreads();

  // ---- (2) the r largest eigenvalues: Gershgorin interval, then multisection on Sturm counts ----
  if (wave == 0) {
    double lo = 1e300, hi = -1e300, em = 0.;
    for (int i = lane; i < n; i += 64) {
      const double rad = (i > 0 ? fabs(se[i - 1]) : 0.) + (i + 1 < n ? fabs(se[i]) : 0.);
      lo = fmin(lo, sd[i] - rad);
      hi = fmax(hi, sd[i] + rad);
      em = fmax(em, se2[i]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      lo = fmin(lo, __shfl_xor(lo, off, 64));
      hi = fmax(hi, __shfl_xor(hi, off, 64));
      em = fmax(em, __shfl_xor(em, off, 64));
    }
    if (lane == 0) {
      const double tn = fmax(fabs(lo), fabs(hi));
      const double pivmin = 2.2250738585072014e-308 * fmax(1., em);
      const double slack = 2.1 * tn * 2.220446049250313e-16 * n + 2.1 * pivmin;
      s_gl = lo - slack;
      s_gu = hi + slack;
      s_pivmin = pivmin;
    }
  }
  __syncthreads();
  const double pivmin = s_pivmin;
  const double tnorm = fmax(fabs(s_gl), fabs(s_gu));
  {
    const int g = tid >> 5, j = tid & 31;
    for (int kk = g; kk < r; kk += kTridThreads / 32) {
      const int kasc = n - 1 - kk;                 // kk-th largest = kasc-th smallest (0-based)
      double lo = s_gl, hi = s_gu;
      for (int step = 0; step < kMultiSteps; ++step) {
        const double h = (hi - lo) / 33.;
        const double x = lo + (j + 1) * h;
        const bool above = sturm_count(sd, se2, n, x, pivmin) > kasc;     // more than kasc eigenvalues below x
        const uint64_t bal = __ballot(above);
        const uint32_t mk = (uint32_t)(bal >> (lane & 32));
        // first point with `above`: the eigenvalue lies between it and the point before
        const int jf = mk ? __builtin_ctz(mk) : 32;
        const double nlo = jf == 0 ? lo : lo + jf * h;
        const double nhi = jf == 32 ? hi : lo + (jf + 1) * h;
        lo = nlo;
        hi = nhi;
      }
      if (j == 0) slam[kk] = 0.5 * (lo + hi);
    }
  }
  __syncthreads();
  // close eigenvalues: decline
  if (tid == 0) {
    const double delta = kClusterTol * tnorm;
    int bad = 0;
    for (int k = 0; k < r; ++k) {
      if (!(fabs(slam[k]) <= 1e300)) bad = 1;                          // NaN / inf
      if (k + 1 < r && !(slam[k] - slam[k + 1] >= delta)) bad = 1;
    }
    if (!bad && r < n && sturm_count(sd, se2, n, slam[r - 1] - delta, pivmin) != n - r) bad = 1;
    if (!(tnorm > 0.)) bad = 1;                                         // zero matrix
    s_decline = bad;
    jb.status[0] = 0;
    jb.status[1] = 0;
    jb.status[2] = bad;
  }
  __syncthreads();
  if (s_decline) return;

  // ---- (3) inverse iteration, kInvBatch eigenvectors at a time, one thread each ----
  double* pivA = reinterpret_cast<double*>(T);     // [i][t]: reciprocal pivots of the elimination
  double* U1 = pivA + n * kInvBatch;               //         first super-diagonal of the upper factor
  double* Y = U1 + n * kInvBatch;                  //         right-hand side after the forward sweep
  double* Zv = Y + n * kInvBatch;                  //         current iterate
  double* Zg = trid_Z(jb);
  const double tol = 2.220446049250313e-16 * tnorm;
  for (int b0 = 0; b0 < r; b0 += kInvBatch) {
    const int t = tid;
    if (t < kInvBatch && b0 + t < r) {
      const int k = b0 + t;
      const double lam = slam[k];
      for (int i = 0; i < n; ++i) {
        const uint32_t u = trid_mix((uint32_t)i * 0x9E3779B9u + (uint32_t)k * 0x85EBCA6Bu + 0x1234567u);
        Zv[i * kInvBatch + t] = (double)u * (1. / 2147483648.) - 1.;
      }
      for (int it = 0; it < 3; ++it) {
        uint64_t pv_lo = 0ull, pv_hi = 0ull;                           // bit i: rows interchanged at step i
        // forward: elimination with partial pivoting and the forward substitution in one sweep
        double a = sd[0] - lam, du = se[0], y = Zv[t];
        for (int i = 0; i + 1 < n; ++i) {
          const double sub = se[i], dn = sd[i + 1] - lam, en = i + 2 < n ? se[i + 1] : 0.;
          const double rhs = Zv[(i + 1) * kInvBatch + t];
          if (fabs(a) >= fabs(sub)) {
            if (a == 0.) a = tol;
            const double ra = rcp_nr(fabs(a) < tol ? (a < 0. ? -tol : tol) : a);
            const double f = sub * ra;
            pivA[i * kInvBatch + t] = ra;                              // reciprocal pivots: the back substitution multiplies
            U1[i * kInvBatch + t] = du;
            Y[i * kInvBatch + t] = y;
            a = dn - f * du;
            du = en;
            y = rhs - f * y;
          } else {
            const double rs = rcp_nr(sub);                             // |sub| > |a| >= 0
            const double f = a * rs;
            if (i < 64) pv_lo |= 1ull << i; else pv_hi |= 1ull << (i - 64);
            pivA[i * kInvBatch + t] = fabs(sub) < tol ? (sub < 0. ? -1. / tol : 1. / tol) : rs;
            U1[i * kInvBatch + t] = dn;
            Y[i * kInvBatch + t] = rhs;
            a = du - f * dn;
            du = -f * en;
            y = y - f * rhs;
          }
        }
        if (fabs(a) < tol) a = a < 0. ? -tol : tol;
        pivA[(n - 1) * kInvBatch + t] = rcp_nr(a);
        Y[(n - 1) * kInvBatch + t] = y;
        // backward substitution; second super-diagonal: e[i + 1] where rows were interchanged
        double z1 = 0., z2 = 0., zmax = 0.;
        for (int i = n - 1; i >= 0; --i) {
          const double rp = pivA[i * kInvBatch + t];
          double sacc = Y[i * kInvBatch + t];
          if (i + 1 < n) sacc -= U1[i * kInvBatch + t] * z1;
          const bool swapped = i < 64 ? ((pv_lo >> i) & 1ull) : ((pv_hi >> (i - 64)) & 1ull);
          if (i + 2 < n && swapped) sacc -= se[i + 1] * z2;
          const double z = sacc * rp;
          Zv[i * kInvBatch + t] = z;
          zmax = fmax(zmax, fabs(z));
          z2 = z1;
          z1 = z;
        }
        const double sc = zmax > 0. ? 1. / zmax : 1.;
        for (int i = 0; i < n; ++i) Zv[i * kInvBatch + t] *= sc;
      }
      double nrm2 = 0.;
      for (int i = 0; i < n; ++i) nrm2 += Zv[i * kInvBatch + t] * Zv[i * kInvBatch + t];
      const double inv = nrm2 > 0. ? rsqrt(nrm2) : 0.;
      for (int i = 0; i < n; ++i) Zg[(size_t)k * n + i] = Zv[i * kInvBatch + t] * inv;
    }
    __syncthreads();
  }
}

// (4) U[:, k] = H_0 H_1 .. H_{n-2} z_k, the phase convention and the float32 factor: one wavefront per
// eigenvector, the vector in registers (rows lane and lane + 64), the reflectors read kAheadRefl ahead.
constexpr int kAheadRefl = 4;
__global__ __launch_bounds__(64) void k_trid_back(EigJobs jobs) {
  const EigJob jb = jobs.job[blockIdx.y];
  const int n = jb.n, r = jb.r;
  const int k = blockIdx.x;
  if (k >= r || jb.status[2] != 0) return;
  const int lane = threadIdx.x;
  const double2* Vg = reinterpret_cast<const double2*>(jb.V);
  const double2* tauG = trid_tau(jb);
  const double* Zg = trid_Z(jb);
  const int r0 = lane, r1 = lane + 64;
  double2 x0 = make_double2(r0 < n ? Zg[(size_t)k * n + r0] : 0., 0.);
  double2 x1 = make_double2(r1 < n ? Zg[(size_t)k * n + r1] : 0., 0.);
  double2 pv0[kAheadRefl], pv1[kAheadRefl], ptau[kAheadRefl];
  auto issue = [&](int i, int slot) {
    const double2 zero = make_double2(0., 0.);
    const int ic = i >= 0 ? i : 0;
    ptau[slot] = tauG[ic];
    pv0[slot] = (i >= 0 && r0 > i && r0 < n) ? Vg[(size_t)ic * n + r0] : zero;
    pv1[slot] = (i >= 0 && r1 > i && r1 < n) ? Vg[(size_t)ic * n + r1] : zero;
  };
#pragma unroll
  for (int d = 0; d < kAheadRefl; ++d) issue(n - 2 - d, d);
  for (int base = n - 2; base >= 0; base -= kAheadRefl) {
#pragma unroll
    for (int d = 0; d < kAheadRefl; ++d) {
      const int i = base - d;
      const double2 tau = ptau[d], v0 = pv0[d], v1 = pv1[d];
      issue(i - kAheadRefl, d);
      if (i >= 0) {
        const double2 t0 = cmuld(conjd(v0), x0), t1 = cmuld(conjd(v1), x1);
        const double dx = wave_sum_d(t0.x + t1.x), dy = wave_sum_d(t0.y + t1.y);
        const double2 sfac = cmuld(tau, make_double2(dx, dy));
        const double2 u0 = cmuld(sfac, v0), u1 = cmuld(sfac, v1);
        x0 = make_double2(x0.x - u0.x, x0.y - u0.y);
        x1 = make_double2(x1.x - u1.x, x1.y - u1.y);
      }
    }
  }
  // unit phase that makes the largest-modulus entry (lowest row on ties) real and positive
  double best = r0 < n ? x0.x * x0.x + x0.y * x0.y : -1.;
  int brow = r0;
  double2 bval = x0;
  {
    const double a1 = r1 < n ? x1.x * x1.x + x1.y * x1.y : -1.;
    if (a1 > best) { best = a1; brow = r1; bval = x1; }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const double ob = __shfl_xor(best, off, 64);
    const int orow = __shfl_xor(brow, off, 64);
    const double ovx = __shfl_xor(bval.x, off, 64), ovy = __shfl_xor(bval.y, off, 64);
    if (ob > best || (ob == best && orow < brow)) { best = ob; brow = orow; bval = make_double2(ovx, ovy); }
  }
  const double mag = sqrt(best);
  const double2 ph = mag > 0. ? make_double2(bval.x / mag, -bval.y / mag) : make_double2(1., 0.);
  float2* U = reinterpret_cast<float2*>(jb.U);
  if (r0 < n) {
    const double2 v = cmuld(x0, ph);
    U[(size_t)r0 * r + k] = make_float2((float)v.x, (float)v.y);
  }
  if (r1 < n) {
    const double2 v = cmuld(x1, ph);
    U[(size_t)r1 * r + k] = make_float2((float)v.x, (float)v.y);
  }
}

__global__ void k_identity_factor(float2* U, int n) {
  int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n * n) U[e] = make_float2((e / n) == (e % n) ? 1.f : 0.f, 0.f);
}

}  // namespace

// Bytes of the per-mode work buffer `work_a` of launch_eig_batch: the work matrix for the
// memory-resident solver, header + rotation log (every round of every sweep) for the LDS solver.
size_t eig_work_bytes(int n) {
  if (n > kEigTriMaxN) return (size_t)n * n * sizeof(double2);
  const int m = n + (n & 1);
  return sizeof(EigLogHeader) + (size_t)kEigMaxSweeps * (m - 1) * (m / 2) * sizeof(RotLog);
}

int gram_num_chunks(int64_t A, int In, int64_t B) {
  (void)In;
  const int64_t J = A * B;
  const int64_t tiles = (J + kTC - 1) / kTC;
  return (int)(tiles < 256 ? (tiles < 1 ? 1 : tiles) : 256);
}

void launch_gram(hipStream_t s, const void* g, int dtype, const uint32_t* mask, int64_t A, int In,
                 int64_t B, int nchunks, double* partials) {
  const int64_t J = A * B;
  const int64_t tiles = (J + kTC - 1) / kTC;
  const int64_t tiles_per_chunk = (tiles + nchunks - 1) / nchunks;
  const int64_t cols_per_chunk = tiles_per_chunk * kTC;
  const int nsup = (In + kSuper - 1) / kSuper;
  const size_t lds = (size_t)2 * kSuper * kRowD * sizeof(double);   // 132 KB: more than the default limit
  // One super block (every FNO extent) and lane offsets that fit 32 bits: the kernel with the lean fetch.
  // Its offsets reach two leading indices ahead: 2 In B elements of at most 8 bytes.
  if (nsup == 1 && (int64_t)In * B < ((int64_t)1 << 28)) {
    dim3 grid((unsigned)nchunks), block(kGram128Threads);
    const bool smallb = B < kTC;
    const uint32_t magic = B <= 1 ? 0u : (uint32_t)((0x100000000ull + (uint64_t)B - 1) / (uint64_t)B);
#define TGRAD_GRAM128(DT_, SB_)                                                                         \
  do {                                                                                                  \
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_gram128<DT_, SB_>),                       \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                    \
    k_gram128<DT_, SB_><<<grid, block, lds, s>>>(g, mask, A, In, B, cols_per_chunk, magic, partials);   \
  } while (0)
    if (dtype == TGRAD_C64) { if (smallb) TGRAD_GRAM128(TGRAD_C64, true); else TGRAD_GRAM128(TGRAD_C64, false); }
    else { if (smallb) TGRAD_GRAM128(TGRAD_CBF16, true); else TGRAD_GRAM128(TGRAD_CBF16, false); }
#undef TGRAD_GRAM128
    return;
  }
  dim3 grid((unsigned)nchunks, (unsigned)(nsup * nsup)), block(kGramThreads);
  if (dtype == TGRAD_C64) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_gram<TGRAD_C64>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    k_gram<TGRAD_C64><<<grid, block, lds, s>>>(g, mask, A, In, B, cols_per_chunk, partials);
  } else {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_gram<TGRAD_CBF16>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    k_gram<TGRAD_CBF16><<<grid, block, lds, s>>>(g, mask, A, In, B, cols_per_chunk, partials);
  }
}

void launch_gram_reduce(hipStream_t s, const double* partials, int nchunks, int In, double* gram) {
  const int64_t n2 = (int64_t)In * In;
  k_gram_reduce<<<dim3((unsigned)((n2 + kReduceElems - 1) / kReduceElems)), dim3(256), 0, s>>>(partials, nchunks, In,
                                                                                          gram);
}

void launch_eig_batch(hipStream_t s, int njobs, const double* const* gram, double* const* work_a,
                      double* const* work_v, const int* In, const int* r, float* const* U, int* const* status,
                      int max_sweeps) {
  // max_sweeps == 0: the tridiagonal path first, Jacobi (full sweep budget) where it declines;
  // 1 .. kEigMaxSweeps: Jacobi with that budget for every solve
  const int use_fast = max_sweeps <= 0 ? 1 : 0;
  if (max_sweeps <= 0 || max_sweeps > kEigMaxSweeps) max_sweeps = kEigMaxSweeps;   // the log is sized for kEigMaxSweeps
  if (njobs <= 0) return;
  EigJobs small, large;                          // n <= 128: work matrix in LDS; larger: in memory
  int nsmall = 0, nlarge = 0, nmax = 0;
  for (int i = 0; i < njobs; ++i) {
    EigJob jb;
    jb.gram = gram[i];
    jb.A = work_a[i];
    jb.V = work_v[i];
    jb.U = U[i];
    jb.status = status[i];
    jb.n = In[i];
    jb.r = r[i];
    jb.max_sweeps = max_sweeps;
    jb.use_fast = In[i] <= kEigTriMaxN ? use_fast : 0;
    if (In[i] <= kEigTriMaxN) {
      small.job[nsmall++] = jb;
      if (In[i] > nmax) nmax = In[i];
    } else {
      large.job[nlarge++] = jb;
    }
  }
  if (nsmall > 0) {
    const size_t lds = (size_t)nmax * (nmax + 1) / 2 * sizeof(double2);
    static bool attr_set = false;
    if (!attr_set) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_eig_tri), hipFuncAttributeMaxDynamicSharedMemorySize,
                                kEigTriMaxN * (kEigTriMaxN + 1) / 2 * (int)sizeof(double2));
      attr_set = true;
    }
    if (use_fast) {
      int rmax = 1;
      for (int i = 0; i < nsmall; ++i) rmax = small.job[i].r > rmax ? small.job[i].r : rmax;
      const size_t inv = (size_t)4 * nmax * kInvBatch * sizeof(double);
      const size_t lds_t = lds > inv ? lds : inv;
      static bool attr_t = false;
      if (!attr_t) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_trid), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  kEigTriMaxN * (kEigTriMaxN + 1) / 2 * (int)sizeof(double2));
        attr_t = true;
      }
      k_trid<<<dim3((unsigned)nsmall), dim3(kTridThreads), lds_t, s>>>(small);
      k_trid_back<<<dim3((unsigned)rmax, (unsigned)nsmall), dim3(64), 0, s>>>(small);
    }
    k_eig_tri<<<dim3((unsigned)nsmall), dim3(kEigThreads), lds, s>>>(small);
    k_eig_apply<<<dim3((unsigned)nmax, (unsigned)nsmall), dim3(64), 0, s>>>(small);
    k_eig_finish<<<dim3((unsigned)nsmall), dim3(kEigThreads), 0, s>>>(small);
  }
  if (nlarge > 0) k_eig<<<dim3((unsigned)nlarge), dim3(kEigThreads), 0, s>>>(large);
}

void launch_identity_factor(hipStream_t s, float* U, int n) {
  k_identity_factor<<<dim3((unsigned)((n * n + 255) / 256)), dim3(256), 0, s>>>(
      reinterpret_cast<float2*>(U), n);
}

}  // namespace tgrad
