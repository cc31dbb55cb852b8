// Mode-n products of the per-step path of Algorithm 1 on the fp32 matrix cores
// (v_mfma_f32_32x32x2f32), for low-rank compression  g_L = (G - Sparse(G, Omega)) x_n U^(n)H
// and reconstruction  G~_L = N_L x_n U^(n)  (section "Low-rank gradient tensor decomposition",
// appendix "Tensor Operations and Notation", mode-k product).
//
// A complex contraction is run as a real one without padding or wasted flops: a tensor of
// interleaved (re, im) float32 pairs is used as it lies in memory, and the factor is expanded to
// its 2 x 2 real blocks.  With F = Fr + i Fi and X = Xr + i Xi,
//   re(F X) = Fr Xr - Fi Xi,   im(F X) = Fr Xi + Fi Xr,
// i.e. 4 real multiply-adds per complex multiply-add on either layout below.
//
// The kernels:
//  k_mid      contracts a mode that is NOT the last one: the tensor is (A, K, B) with B >= 1
//             contiguous; every lane owns VEC complex columns (a, b) and walks the K rows.
//  k_core     mode 1 both ways around AdamUpdate on the Tucker core, in one launch.
//  k_core2    modes 1 and 2 both ways around AdamUpdate on the core, one workgroup per column group:
//             everything between the two fused end kernels of a four-way tensor, in one launch.
//  k_lproj    contracts the LAST mode of the gradient itself (first compression stage): a
//             flat tile of rows is staged in LDS, the entries of the support Omega that fall
//             in the tile are handed to the sparse branch (gather) and zeroed (this is
//             G - Sparse(G, Omega) without a second pass over G), then 32 rows per wavefront
//             go through the matrix cores.  With FUSE it also contracts mode N-1 (the tile's mode-N
//             result, still in the accumulators, is the operand of the next contraction);
//             k_lproj_flat is that fused form for odd last extents.
//  k_lupdate  the last reconstruction stage fused with everything that touches W: expands the
//             last mode into an LDS tile, runs AdamUpdate on the sparse values of the tile
//             and adds lambda N_S into it, then streams W <- W (1 - lr wd) - lr tile with
//             16-byte accesses.  k_lupdate_fused also expands mode N-1 in front of it.
//  k_mfma_probe_*  register-resident matrix-core loops (calibration of the reported fractions).
//
// Operand layout of v_mfma_f32_32x32x2f32 (D = A B + C, A 32 x 2, B 2 x 32, 64 lanes):
//   lane l supplies A[l % 32][l / 32] and B[l / 32][l % 32];
//   register r of lane l receives D[(r % 4) + 8 (r / 4) + 4 (l / 32)][l % 32].
#include <atomic>
#include <map>
#include <mutex>
#include <type_traits>
#include <utility>

#include "device_common.h"

namespace tgrad {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ v16f mfma32(float a, float b, v16f c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ int d_row(int r, int half) { return (r & 3) + 8 * (r >> 2) + 4 * half; }

// q = n / d, exact for n * d < 2^32 (callers keep n < 2^17, d < 2^10).
// magic = ceil(2^32 / d); d == 1 is encoded as magic == 0.
__device__ __forceinline__ uint32_t div_magic(uint32_t n, uint32_t magic) {
  return magic ? __umulhi(n, magic) : n;
}

// -------------------------------------------------------------------------------------------
// Register-resident matrix-core loops: what the matrix cores of this chip deliver when nothing else
// is in the way (no memory, no LDS, operands constant).  The reference point for the matrix-core
// fractions of the kernels below, next to the published peaks.  Four independent accumulators per
// wavefront, two wavefronts per SIMD.
typedef double v4d __attribute__((ext_vector_type(4)));
constexpr int kProbeChains = 4;
constexpr int kProbeUnroll = 64;             // rounds per trip of the loop (the loop's own bookkeeping is then negligible)
__global__ __launch_bounds__(256) void k_mfma_probe_f32(float* sink, int64_t iters, float a, float b) {
  v16f acc[kProbeChains];
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  for (int64_t i = 0; i < iters; i += kProbeUnroll) {          // (iters is a multiple of kProbeUnroll: host)
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u)
#pragma unroll
      for (int c = 0; c < kProbeChains; ++c) acc[c] = mfma32(a, b, acc[c]);
  }
  float t = 0.f;
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) t += acc[c][r];
  if (t == 12345.678f) sink[0] = t;                            // (never: a b iters is not that number; keeps the loop alive)
}
__global__ __launch_bounds__(256) void k_mfma_probe_f64(float* sink, int64_t iters, double a, double b) {
  v4d acc[kProbeChains];
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[c][r] = 0.;
  for (int64_t i = 0; i < iters; i += kProbeUnroll) {
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u)
#pragma unroll
      for (int c = 0; c < kProbeChains; ++c) acc[c] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[c], 0, 0, 0);
  }
  double t = 0.;
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int r = 0; r < 4; ++r) t += acc[c][r];
  if (t == 12345.678) sink[0] = (float)t;
}

// -------------------------------------------------------------------------------------------
// k_mid: out[a, m, b] = sum_k F[m, k] x[a, k, b],  F = U^H (PROJECT) or U.
// Workgroup = 4 wavefronts; a wavefront owns 32 column vectors (VEC complex each) and MT row
// tiles of 32 output rows; blockIdx.y selects the group of MT row tiles.
// Per pair of rows (k = 2 j, 2 j + 1): lanes 0..31 load row 2 j, lanes 32..63 row 2 j + 1 of
// their column; the factor operands (Fr, Fi) for that pair come from LDS.
constexpr int kMidThreads = 256;
constexpr int kMidJChunk = 64;            // row pairs of the factor staged in LDS at a time
constexpr int kMidUnroll = 8;

// Fills dst[0 .. total) with gen(e), `kStageBatch` global loads per thread in flight at a time (a
// plain loop would pay one memory round trip per element and thread).
constexpr int kStageBatch = 8;
template <typename Gen>
__device__ __forceinline__ void stage_batched(float2* dst, int total, int tid, int nthreads, Gen gen) {
  for (int e0 = tid; e0 < total; e0 += nthreads * kStageBatch) {
    float2 f[kStageBatch];
#pragma unroll
    for (int u = 0; u < kStageBatch; ++u) {
      const int e = e0 + u * nthreads;
      f[u] = gen(e < total ? e : total - 1);
    }
#pragma unroll
    for (int u = 0; u < kStageBatch; ++u) {
      const int e = e0 + u * nthreads;
      if (e < total) dst[e] = f[u];
    }
  }
}

template <int VEC> struct VecT;
template <> struct VecT<1> { typedef float2 type; };
template <> struct VecT<2> { typedef float4 type; };

// MODE 0: every wavefront of a workgroup owns its own 32 column vectors and all MT row tiles.
// MODE 1 (split-K, MT = 1): the 4 wavefronts share 32 column vectors and deal the row pairs
//         round-robin; their partial tiles are summed through LDS in a fixed order.  For stages
//         with few columns, where MODE 0 would leave most of the chip idle.
// MODE 2 (MT = 1): the 4 wavefronts share 32 column vectors and own one 32-row output tile each
//         (128 output rows per workgroup).  For reconstruction stages with few columns.
template <int MT, int VEC, bool PROJECT, int MODE>
__global__ __launch_bounds__(kMidThreads) void k_mid(const float* __restrict__ x,
                                                     const float2* __restrict__ U, int rn, int64_t A,
                                                     int K, int M, int64_t B, float* __restrict__ out) {
  typedef typename VecT<VEC>::type V;
  constexpr int TL = MODE == 2 ? 4 : MT;  // row tiles whose factor operands a workgroup stages
  extern __shared__ float2 sF[];          // [pair][tile][lane] = (Fr, Fi)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int64_t BV = B / VEC;             // host guarantees B % VEC == 0
  const int64_t ncv = A * BV;
  const int64_t cv_raw = MODE == 0 ? ((int64_t)blockIdx.x * (kMidThreads / 64) + wave) * 32 + col
                                   : (int64_t)blockIdx.x * 32 + col;
  const bool valid = cv_raw < ncv;
  const int64_t cv = valid ? cv_raw : ncv - 1;   // lanes past the end load a real column, store nothing
  const int64_t a = cv / BV;
  const int64_t bv = cv - a * BV;
  const float* xp = x + ((a * K) * B + bv * VEC) * 2;
  const int64_t row_stride = B * 2;       // floats between consecutive k
  const int mbase = blockIdx.y * (32 * TL);
  const int my_tile0 = MODE == 2 ? wave : 0;   // first of this wavefront's MT tiles among the staged TL

  v16f acc[MT][2 * VEC];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < 2 * VEC; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][t][r] = 0.f;

  // One row pair: lanes 0..31 hold row 2 j, lanes 32..63 row 2 j + 1 of their column.  The loads are
  // unconditional (a row index past K is clamped to the last row: its factor operands are zero), and
  // the loops below carry no guards: predicated loads and guarded MFMAs both stall the pipeline.
  auto load_pair_row = [&](int j) -> V {
    const int k = 2 * j + half;
    return *reinterpret_cast<const V*>(xp + (int64_t)(k < K ? k : K - 1) * row_stride);
  };
  auto mfma_pair_row = [&](const V& v, int jj) {
    float xs[2 * VEC], xj[2 * VEC];
    if constexpr (VEC == 1) {
      xs[0] = v.x; xs[1] = v.y;
    } else {
      xs[0] = v.x; xs[1] = v.y; xs[2] = v.z; xs[3] = v.w;
    }
#pragma unroll
    for (int c = 0; c < VEC; ++c) {                            // (X J): re column <- -im, im column <- re
      xj[2 * c] = -xs[2 * c + 1];
      xj[2 * c + 1] = xs[2 * c];
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const float2 f = sF[(jj * TL + my_tile0 + mt) * 64 + lane];
#pragma unroll
      for (int t = 0; t < 2 * VEC; ++t) {
        acc[mt][t] = mfma32(f.x, xs[t], acc[mt][t]);
        acc[mt][t] = mfma32(f.y, xj[t], acc[mt][t]);
      }
    }
  };

  constexpr int JSTEP = MODE == 1 ? 4 : 1;                     // split-K: wavefront w takes pairs w, w + 4, ...
  const int jfirst = MODE == 1 ? wave : 0;
  const int J = (K + 1) >> 1;
  for (int jc0 = 0; jc0 < J; jc0 += kMidJChunk) {
    const int jn = (J - jc0) < kMidJChunk ? (J - jc0) : kMidJChunk;
    // the chunk's first batch of rows goes in flight before the factor operands are staged
    V cur[kMidUnroll];
#pragma unroll
    for (int u = 0; u < kMidUnroll; ++u) cur[u] = load_pair_row(jc0 + jfirst + u * JSTEP);
    __syncthreads();                                           // previous chunk fully consumed
    stage_batched(sF, jn * TL * 64, tid, kMidThreads, [&](int e) -> float2 {
      const int l = e & 63;
      const int mt = (e >> 6) % TL;
      const int jj = e / (64 * TL);
      const int m = mbase + 32 * mt + (l & 31);
      const int k = 2 * (jc0 + jj) + (l >> 5);
      const bool in = m < M && k < K;                          // outside: a clamped, valid element times zero
      const int mc = in ? m : 0, kc = in ? k : 0;
      const float2 u = PROJECT ? U[(int64_t)kc * rn + mc] : U[(int64_t)mc * rn + kc];
      return in ? make_float2(u.x, PROJECT ? -u.y : u.y) : make_float2(0.f, 0.f);
    });
    __syncthreads();
    // Row pairs in batches of kMidUnroll, the next batch's loads issued before the current batch
    // goes to the matrix cores (rows past the end are clamped onto the last one and not used).
    int jj = jfirst;
    for (; jj + (kMidUnroll - 1) * JSTEP < jn; jj += kMidUnroll * JSTEP) {
      V nxt[kMidUnroll];
#pragma unroll
      for (int u = 0; u < kMidUnroll; ++u) nxt[u] = load_pair_row(jc0 + jj + (kMidUnroll + u) * JSTEP);
#pragma unroll
      for (int u = 0; u < kMidUnroll; ++u) mfma_pair_row(cur[u], jj + u * JSTEP);
#pragma unroll
      for (int u = 0; u < kMidUnroll; ++u) cur[u] = nxt[u];
    }
#pragma unroll
    for (int u = 0; u < kMidUnroll; ++u)
      if (jj + u * JSTEP < jn) mfma_pair_row(cur[u], jj + u * JSTEP);
  }
  if constexpr (MODE == 1) {
    // partial tiles of wavefronts 1..3 -> LDS, summed by wavefront 0 in a fixed order
    __syncthreads();                                           // factor operands no longer needed
    float* red = reinterpret_cast<float*>(sF);                 // [wave - 1][t][r][lane]
    if (wave > 0) {
#pragma unroll
      for (int t = 0; t < 2 * VEC; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[(((wave - 1) * 2 * VEC + t) * 16 + r) * 64 + lane] = acc[0][t][r];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll 1
    for (int w = 0; w < 3; ++w)
#pragma unroll
      for (int t = 0; t < 2 * VEC; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][t][r] += red[((w * 2 * VEC + t) * 16 + r) * 64 + lane];
  }
  if (!valid) return;
  float* op = out + ((a * M) * B + bv * VEC) * 2;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = mbase + 32 * (my_tile0 + mt) + d_row(r, half);
      if (m < M) {
        float* o = op + (int64_t)m * row_stride;
        if constexpr (VEC == 1) {
          *reinterpret_cast<float2*>(o) = make_float2(acc[mt][0][r], acc[mt][1][r]);
        } else {
          *reinterpret_cast<float4*>(o) = make_float4(acc[mt][0][r], acc[mt][1][r], acc[mt][2][r], acc[mt][3][r]);
        }
      }
    }
}

// -------------------------------------------------------------------------------------------
// k_core: the three steps around the Tucker core in one kernel, for mode 1 (the slowest index):
//   g_L[m, b] = sum_k conj(U[k, m]) x[k, b]            last compression stage (K = I_1, M = r_1 <= 32)
//   N_L = AdamUpdate(g_L)                               appendix algorithm "Adam with low-rank tensor
//                                                       decomposition" (moments updated in place)
//   z[i, b]   = sum_m U[i, m] N_L[m, b]                 first reconstruction stage
// so the core gradient and the core update never travel through memory between kernels (g_L is
// still written out: it is part of the readable state).
// A workgroup of 4 wavefronts owns 32 column vectors (VEC complex each).  Compression is split over
// the wavefronts by row pairs (wavefront w takes pairs w, w + 4, ...) and summed through LDS in a
// fixed order; every wavefront runs AdamUpdate on a quarter of the 32 x 32 VEC tile and hands its
// part of N_L back through LDS; then wavefront w expands the output row tiles w, w + 4, ...  The accumulator registers of the
// compression ARE the B operands of the expansion: register r of lane (col, half) holds row
// m = d_row(r, half), so expansion step r pairs rows d_row(r, 0) and d_row(r, 1) and its factor
// operand is U[i, d_row(r, half)].
// `z` may be `x` (in place): a workgroup writes only the columns it alone has read, and its reads
// are complete (workgroup barriers in between) before its first write.
struct CoreAdam {
  float2* m;            // first moments, (M, B) complex
  float* v;             // second moments
  float2* g_out;        // compressed gradient, written for the state accessors
  float beta1, beta2, inv_c1, inv_c2, eps;
};

template <int VEC>
__global__ __launch_bounds__(kMidThreads) void k_core(const float* x, const float2* __restrict__ U,
                                                      int rn, int K, int M, int64_t B, CoreAdam ad,
                                                      float* z) {
  typedef typename VecT<VEC>::type V;
  constexpr int NT = 2 * VEC;                   // accumulator tiles: (column of the vector, re / im)
  extern __shared__ float2 sF[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  const int64_t BV = B / VEC;
  const int64_t cv_raw = (int64_t)blockIdx.x * 32 + col;
  const bool valid = cv_raw < BV;
  const int64_t cv = valid ? cv_raw : BV - 1;
  const int64_t row_stride = B * 2;
  const float* xp = x + cv * VEC * 2;
  const int J = (K + 1) >> 1;                   // row pairs of the compression
  const int NTI = (K + 31) >> 5;                // output row tiles of the expansion
  // LDS: [0, J*64) compression operands, reused afterwards for the reduction / hand-over buffer;
  //      then 16 * NTI * 64 expansion operands
  float2* sFp = sF;
  const int red_f2 = 4 * NT * 16 * 64 / 2;                       // float2 slots of the reduction buffer
  float2* sFe = sF + (J * 64 > red_f2 ? J * 64 : red_f2);
  stage_batched(sFp, J * 64, tid, kMidThreads, [&](int e) -> float2 {
    const int l = e & 63, jj = e >> 6;
    const int m = l & 31, k = 2 * jj + (l >> 5);
    const bool in = m < M && k < K;
    const float2 u = U[in ? (int64_t)k * rn + m : 0];
    return in ? make_float2(u.x, -u.y) : make_float2(0.f, 0.f);
  });
  stage_batched(sFe, 16 * NTI * 64, tid, kMidThreads, [&](int e) -> float2 {
    const int l = e & 63, mt = (e >> 6) % NTI, r = e / (64 * NTI);
    const int i = 32 * mt + (l & 31), m = d_row(r, l >> 5);
    const bool in = i < K && m < M;
    const float2 u = U[in ? (int64_t)i * rn + m : 0];
    return in ? u : make_float2(0.f, 0.f);
  });
  __syncthreads();

  v16f acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
  auto load_pair_row = [&](int j) -> V {
    const int k = 2 * j + half;
    return *reinterpret_cast<const V*>(xp + (int64_t)(k < K ? k : K - 1) * row_stride);
  };
  auto mfma_pair_row = [&](const V& v, int jj) {
    float xs[NT], xj[NT];
    if constexpr (VEC == 1) {
      xs[0] = v.x; xs[1] = v.y;
    } else {
      xs[0] = v.x; xs[1] = v.y; xs[2] = v.z; xs[3] = v.w;
    }
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      xj[2 * c] = -xs[2 * c + 1];
      xj[2 * c + 1] = xs[2 * c];
    }
    const float2 f = sFp[jj * 64 + lane];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      acc[t] = mfma32(f.x, xs[t], acc[t]);
      acc[t] = mfma32(f.y, xj[t], acc[t]);
    }
  };
  {
    constexpr int kAhead = 16;                                 // row pairs in flight: all of them for K <= 128
    int jj = wave;
    for (; jj + (kAhead - 1) * 4 < J; jj += kAhead * 4) {
      V v[kAhead];
#pragma unroll
      for (int u = 0; u < kAhead; ++u) v[u] = load_pair_row(jj + u * 4);
#pragma unroll
      for (int u = 0; u < kAhead; ++u) mfma_pair_row(v[u], jj + u * 4);
    }
    for (; jj < J; jj += 4) mfma_pair_row(load_pair_row(jj), jj);
  }
  // ---- all partial tiles -> LDS; wavefront w then owns registers r = 4 w .. 4 w + 3 of the tile: it
  //      sums the four partials in a fixed order (wavefront 0's first), runs AdamUpdate on those
  //      core rows and hands N_L back through LDS ----
  __syncthreads();                                             // compression operands no longer needed
  float* red = reinterpret_cast<float*>(sF);                   // [wave][t][r][lane]
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) red[((wave * NT + t) * 16 + r) * 64 + lane] = acc[t][r];
  __syncthreads();
  float2 nn[4][VEC];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r = 4 * wave + q;
    const int m = d_row(r, half);
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      float gre = 0.f, gim = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        gre += red[((w * NT + 2 * c) * 16 + r) * 64 + lane];
        gim += red[((w * NT + 2 * c + 1) * 16 + r) * 64 + lane];
      }
      nn[q][c] = make_float2(0.f, 0.f);
      if (valid && m < M) {
        const int64_t idx = (int64_t)m * B + cv * VEC + c;
        float2 mm = ad.m[idx];
        mm.x = ad.beta1 * mm.x + (1.f - ad.beta1) * gre;
        mm.y = ad.beta1 * mm.y + (1.f - ad.beta1) * gim;
        const float vv = ad.beta2 * ad.v[idx] + (1.f - ad.beta2) * (gre * gre + gim * gim);
        ad.m[idx] = mm;
        ad.v[idx] = vv;
        ad.g_out[idx] = make_float2(gre, gim);
        const float d = 1.f / (sqrtf(vv * ad.inv_c2) + ad.eps);
        nn[q][c] = make_float2(mm.x * ad.inv_c1 * d, mm.y * ad.inv_c1 * d);
      }
    }
  }
  __syncthreads();                                             // every partial has been read
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      red[((2 * c) * 16 + 4 * wave + q) * 64 + lane] = nn[q][c].x;
      red[((2 * c + 1) * 16 + 4 * wave + q) * 64 + lane] = nn[q][c].y;
    }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = red[(t * 16 + r) * 64 + lane];
  // ---- expansion: wavefront w writes output row tiles w, w + 4, ... ----
  float* op = z + cv * VEC * 2;
  for (int mt = wave; mt < NTI; mt += 4) {
    v16f out[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) out[t][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float2 f = sFe[(r * NTI + mt) * 64 + lane];
#pragma unroll
      for (int c = 0; c < VEC; ++c) {
        const float nr = acc[2 * c][r], ni = acc[2 * c + 1][r];
        out[2 * c] = mfma32(f.x, nr, out[2 * c]);
        out[2 * c] = mfma32(f.y, -ni, out[2 * c]);
        out[2 * c + 1] = mfma32(f.x, ni, out[2 * c + 1]);
        out[2 * c + 1] = mfma32(f.y, nr, out[2 * c + 1]);
      }
    }
    if (valid) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = 32 * mt + d_row(r, half);
        if (i < K) {
          float* o = op + (int64_t)i * row_stride;
          if constexpr (VEC == 1) {
            *reinterpret_cast<float2*>(o) = make_float2(out[0][r], out[1][r]);
          } else {
            *reinterpret_cast<float4*>(o) = make_float4(out[0][r], out[1][r], out[2][r], out[3][r]);
          }
        }
      }
    }
  }
}

// -------------------------------------------------------------------------------------------
// k_core2: everything between the fused first projection and the fused update when exactly two
// modes (the two leading ones) are left to compress: y is (I0 = 128, I1, Cc), its Cc complex
// columns contiguous.  Every column c goes through
//   g_L[m0, m1, c] = sum_{i0, i1} conj(U0[i0, m0]) conj(U1[i1, m1]) y[i0, i1, c]   last two compression stages
//   N_L            = AdamUpdate(g_L)                (appendix algorithm "Adam with low-rank tensor decomposition")
//   z[i0, i1, c]   = sum_{m0, m1} U0[i0, m0] U1[i1, m1] N_L[m0, m1, c]             first two reconstruction stages
// on its own, so a workgroup that owns VEC = 2 neighbouring columns (16 bytes per (i0, i1); VEC = 1, 8 bytes,
// where two per workgroup would leave most of the chip without work) runs the whole
// chain between workgroup barriers: nothing travels through memory between the five steps and the
// launches, prologues and tails of three kernels become one.  Wavefront w owns the rows
// i0 = 32 w .. 32 w + 31.  The accumulator layout of one stage is the operand layout of the next
// (register r of lane (col, half) holds row d_row(r, half) of the tile, and a matrix-core step pairs
// exactly the rows d_row(r, 0) and d_row(r, 1)), so no stage transposes anything:
//   1  T[i0, m1]   = sum_i1 y[i0, i1] conj(U1[i1, m1])   data = A operand (lane = i0), U1 from LDS;  D: i0 in registers, m1 in lanes
//   2  P[m0, m1]   = sum_i0 conj(U0[i0, m0]) T[i0, m1]   U0 = A operand, T = B operand straight from the accumulators;
//                                                        the four wavefronts' partial sums meet in LDS, fixed order
//   -  AdamUpdate on the 32 x 32 x VEC core entries of the workgroup's columns, N_L back into LDS in accumulator layout
//   3  R[m1, i0]   = sum_m0 N_L[m0, m1] U0[i0, m0]       N_L = A operand (LDS), U0 = B operand;  D: m1 in registers, i0 in lanes
//   4  z[i0, i1]   = sum_m1 R[m1, i0] U1[i1, m1]         R = A operand straight from the accumulators, U1 from LDS;
//                                                        D: i0 in registers, i1 in lanes
// The factor operands of all four stages come from a table in operand order that is built once per
// refresh (k_pack_core2): the prologue is a straight copy with every load in flight at once.
// The result is written one column group at a time, z[group][i0][i1] in units of VEC complex, because in
// stage 4 neighbouring lanes hold neighbouring i1: the stores of a wavefront are then 512 (256)
// contiguous bytes instead of 64 pieces each in a cache line of its own (the fused update reads its
// operand rows through strides, see FusedPrev).  Workgroups that share cache lines of y (8 column
// pairs per 128 bytes) get consecutive blockIdx / 8, i.e. the same XCD under round-robin dispatch.
struct Core2Args {
  const float* y;       // (128, I1, Cc) complex
  float* z;             // (Cc / G, 128, I1) units of G complex, not the same buffer; G = `zgroup` (2: Cc even)
  const float2* tab;    // core2_table_elems(I1) operands from k_pack_core2
  int I1, M0, M1;
  int64_t Cc;           // a multiple of VEC
  int zgroup;           // columns per unit of z: VEC, or 2 with VEC = 1 (two workgroups then fill a unit)
};
constexpr int kCore2Rows = 128;              // extent of the first mode: 4 wavefronts x 32 rows
constexpr int kCore2Batch = 8;               // row pairs of y per lane in flight (twice that while a batch is computed)

// Operand table: [J1][64] stage 1, [NT1][16][64] stage 4, [4][16][64] stage 2, [4][16][64] stage 3 (float2 each);
// J1 = row pairs of mode 2, NT1 = 32-row tiles of mode 2.
__host__ __device__ inline int core2_table_elems(int I1) { return ((I1 + 1) / 2) * 64 + ((I1 + 31) / 32) * 1024 + 8192; }

__global__ void k_pack_core2(const float2* __restrict__ U0, int rn0, int M0, const float2* __restrict__ U1,
                             int rn1, int M1, int I1, float2* __restrict__ tab) {
  const int J1 = (I1 + 1) >> 1, NT1 = (I1 + 31) >> 5;
  const int n1 = J1 * 64, n4 = NT1 * 1024;
  const int e = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (e >= n1 + n4 + 8192) return;
  const int l = e & 63, col = l & 31, half = l >> 5;
  float2 u = make_float2(0.f, 0.f);
  if (e < n1) {                                    // stage 1: U1[2 j + half][col]
    const int i1 = 2 * (e >> 6) + half;
    if (i1 < I1 && col < M1) u = U1[(int64_t)i1 * rn1 + col];
  } else if (e < n1 + n4) {                        // stage 4: U1[32 tile + col][d_row(r, half)]
    const int q = (e - n1) >> 6, r = q & 15, tile = q >> 4;
    const int i1 = 32 * tile + col, m1 = d_row(r, half);
    if (i1 < I1 && m1 < M1) u = U1[(int64_t)i1 * rn1 + m1];
  } else if (e < n1 + n4 + 4096) {                 // stage 2: U0[32 w + d_row(r, half)][col]
    const int q = (e - n1 - n4) >> 6, r = q & 15, w = q >> 4;
    if (col < M0) u = U0[(int64_t)(32 * w + d_row(r, half)) * rn0 + col];
  } else {                                         // stage 3: U0[32 w + col][d_row(r, half)]
    const int q = (e - n1 - n4 - 4096) >> 6, r = q & 15, w = q >> 4;
    const int m0 = d_row(r, half);
    if (m0 < M0) u = U0[(int64_t)(32 * w + col) * rn0 + m0];
  }
  tab[e] = u;
}

template <int VEC>
__global__ __launch_bounds__(kMidThreads) void k_core2(Core2Args a, CoreAdam ad) {
  typedef typename VecT<VEC>::type V;             // the workgroup's VEC columns of one (i0, i1): 8 or 16 bytes
  constexpr int NT = 2 * VEC;                     // accumulator tiles: (column, re / im)
  extern __shared__ float2 sF[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  const int planes = (int)(a.Cc / VEC);
  const int b = (int)blockIdx.x;
  const int plane = (planes & 7) == 0 ? (b & 7) * (planes >> 3) + (b >> 3) : b;
  const int I1 = a.I1, M0 = a.M0, M1 = a.M1;
  const int J1 = (I1 + 1) >> 1, NT1 = (I1 + 31) >> 5;
  const int64_t row = a.Cc * 2;              // floats between consecutive i1 of y
  const int64_t slab = row * I1;             // floats between consecutive i0 of y
  // LDS: [0, 64 KB) stage-1 operands (J1 x 64 float2), afterwards the partial sums of stage 2
  //      ([wave][t][r][lane] floats) and then N_L ([t][r][lane]); [64 KB, 64 KB + NT1 x 8 KB) stage-4 operands
  float2* sT1 = sF;
  float* red = reinterpret_cast<float*>(sF);
  float2* sT4 = sF + 8192;

  // the first rows of y go in flight, then the stage-1 operands
  const float* xp = a.y + (int64_t)(32 * wave + col) * slab + NT * plane;
  auto load_pair_row = [&](int j) -> V {
    const int jc = j < J1 ? j : J1 - 1;
    const int k = 2 * jc + half;
    return *reinterpret_cast<const V*>(xp + (int64_t)(k < I1 ? k : I1 - 1) * row);
  };
  auto parts = [](const V& v, float* x) {        // x[2 c] = re, x[2 c + 1] = im of column c
    if constexpr (VEC == 1) {
      x[0] = v.x; x[1] = v.y;
    } else {
      x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    }
  };
  V cur[kCore2Batch];
#pragma unroll
  for (int u = 0; u < kCore2Batch; ++u) cur[u] = load_pair_row(u);
  {
    // stage-1 operands -> LDS: 16-byte pieces, 8 per thread (the table holds a multiple of 64 float2)
    const float4* t1 = reinterpret_cast<const float4*>(a.tab);
    float4* d1 = reinterpret_cast<float4*>(sT1);
    const int n1 = J1 * 32;
    float4 p1[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int e = tid + u * kMidThreads;
      p1[u] = t1[e < n1 ? e : 0];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int e = tid + u * kMidThreads;
      if (e < n1) d1[e] = p1[u];
    }
  }
  __syncthreads();
  // What the later stages need travels while stage 1 runs: U0 as the operands of stages 2 and 3
  // (registers) and the moments of this thread's core entries: rows d_row(4 wave + q, half), column col,
  // the workgroup's VEC columns.  (The stage-4 operands travel during stage 2.)
  float2 f2[16], f3[16];
  {
    const float2* t2 = a.tab + J1 * 64 + NT1 * 1024 + wave * 1024 + lane;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      f2[r] = t2[r * 64];
      f3[r] = t2[4096 + r * 64];
    }
  }
  float2 mm[4][VEC];
  float vv[4][VEC];
  int64_t cidx[4];
  bool live[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int m0 = d_row(4 * wave + q, half);
    live[q] = m0 < M0 && col < M1;
    cidx[q] = live[q] ? ((int64_t)m0 * M1 + col) * a.Cc + VEC * plane : 0;
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      mm[q][c] = ad.m[cidx[q] + c];
      vv[q][c] = ad.v[cidx[q] + c];
    }
  }

  // ---- stage 1: T = y conj(U1); tiles (column, re / im) ----
  v16f t[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) t[i][r] = 0.f;
  auto stage1 = [&](const V& v, int j) {
    const float2 f = sT1[j * 64 + lane];
    const float nfy = -f.y;
    float x[NT];
    parts(v, x);
#pragma unroll
    for (int i = 0; i < NT; ++i) t[i] = mfma32(x[i], f.x, t[i]);      // re: yr ur + yi ui;  im: yi ur - yr ui
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      t[2 * c] = mfma32(x[2 * c + 1], f.y, t[2 * c]);
      t[2 * c + 1] = mfma32(x[2 * c], nfy, t[2 * c + 1]);
    }
  };
  {
    int j = 0;
    for (; j + kCore2Batch <= J1; j += kCore2Batch) {
      V nxt[kCore2Batch];
#pragma unroll
      for (int u = 0; u < kCore2Batch; ++u) nxt[u] = load_pair_row(j + kCore2Batch + u);
      __builtin_amdgcn_sched_barrier(0);                       // the loads stay in front of the batch they overlap
#pragma unroll
      for (int u = 0; u < kCore2Batch; ++u) stage1(cur[u], j + u);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < kCore2Batch; ++u) cur[u] = nxt[u];
    }
#pragma unroll
    for (int u = 0; u < kCore2Batch; ++u)
      if (j + u < J1) stage1(cur[u], j + u);
  }
  // ---- stage 2: this wavefront's part of P = conj(U0)^T T over its 32 rows; the stage-4 operands go in flight ----
  const int n4 = NT1 * 512;
  float4 p4[8];
  {
    const float4* t4 = reinterpret_cast<const float4*>(a.tab + J1 * 64);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int e = tid + u * kMidThreads;
      p4[u] = t4[e < n4 ? e : 0];
    }
  }
  v16f p[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) p[i][r] = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const float2 f = f2[r];
    const float nfy = -f.y;
#pragma unroll
    for (int i = 0; i < NT; ++i) p[i] = mfma32(f.x, t[i][r], p[i]);    // re: ur tr + ui ti;  im: ur ti - ui tr
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      p[2 * c] = mfma32(f.y, t[2 * c + 1][r], p[2 * c]);
      p[2 * c + 1] = mfma32(nfy, t[2 * c][r], p[2 * c + 1]);
    }
  }
  {
    float4* d4 = reinterpret_cast<float4*>(sT4);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int e = tid + u * kMidThreads;
      if (e < n4) d4[e] = p4[u];
    }
  }
  __syncthreads();                                             // every wavefront is through with the stage-1 operands
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) red[((wave * NT + i) * 16 + r) * 64 + lane] = p[i][r];
  __syncthreads();
  // ---- AdamUpdate: wavefront w takes registers 4 w .. 4 w + 3 of the tile, partial sums added in wavefront order ----
  float nn[4][NT];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r = 4 * wave + q;
    float g[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      g[i] = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) g[i] += red[((w * NT + i) * 16 + r) * 64 + lane];
    }
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      float2 m = mm[q][c];
      m.x = ad.beta1 * m.x + (1.f - ad.beta1) * g[2 * c];
      m.y = ad.beta1 * m.y + (1.f - ad.beta1) * g[2 * c + 1];
      const float v = ad.beta2 * vv[q][c] + (1.f - ad.beta2) * (g[2 * c] * g[2 * c] + g[2 * c + 1] * g[2 * c + 1]);
      const float d = 1.f / (sqrtf(v * ad.inv_c2) + ad.eps);
      nn[q][2 * c] = nn[q][2 * c + 1] = 0.f;
      if (live[q]) {
        ad.m[cidx[q] + c] = m;
        ad.v[cidx[q] + c] = v;
        ad.g_out[cidx[q] + c] = make_float2(g[2 * c], g[2 * c + 1]);
        nn[q][2 * c] = m.x * ad.inv_c1 * d;
        nn[q][2 * c + 1] = m.y * ad.inv_c1 * d;
      }
    }
  }
  __syncthreads();                                             // every partial sum has been read
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int i = 0; i < NT; ++i) red[(i * 16 + 4 * wave + q) * 64 + lane] = nn[q][i];
  __syncthreads();
  // ---- stage 3: R = N_L^T U0^T for this wavefront's 32 rows i0 ----
  v16f rr[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) rr[i][r] = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const float2 f = f3[r];
    const float nfy = -f.y;
    float n[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) n[i] = red[(i * 16 + r) * 64 + lane];
#pragma unroll
    for (int i = 0; i < NT; ++i) rr[i] = mfma32(n[i], f.x, rr[i]);     // re: nr ur - ni ui;  im: ni ur + nr ui
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      rr[2 * c] = mfma32(n[2 * c + 1], nfy, rr[2 * c]);
      rr[2 * c + 1] = mfma32(n[2 * c], f.y, rr[2 * c + 1]);
    }
  }
  // ---- stage 4: z = R^T U1^T, one tile of 32 columns i1 at a time; z[group][i0][i1], units of zgroup complex ----
  const int ZU = 2 * a.zgroup;                                 // floats per unit
  const int zg = VEC == 1 && a.zgroup == 2 ? plane >> 1 : plane;
  float* zp = a.z + (((int64_t)zg * kCore2Rows + 32 * wave + 4 * half) * I1 + col) * ZU +
              (VEC == 1 && a.zgroup == 2 ? 2 * (plane & 1) : 0);
  for (int tile = 0; tile < NT1; ++tile) {
    v16f z[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) z[i][r] = 0.f;
    const float2* ft = sT4 + tile * 16 * 64 + lane;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float2 f = ft[r * 64];
      const float nfy = -f.y;
#pragma unroll
      for (int c = 0; c < VEC; ++c) {                          // re: rr ur - ri ui;  im: rr ui + ri ur
        z[2 * c] = mfma32(rr[2 * c][r], f.x, z[2 * c]);
        z[2 * c + 1] = mfma32(rr[2 * c][r], f.y, z[2 * c + 1]);
      }
#pragma unroll
      for (int c = 0; c < VEC; ++c) {
        z[2 * c] = mfma32(rr[2 * c + 1][r], nfy, z[2 * c]);
        z[2 * c + 1] = mfma32(rr[2 * c + 1][r], f.x, z[2 * c + 1]);
      }
    }
    if (32 * tile + col < I1) {
      float* zt = zp + 32 * tile * ZU;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float* o = zt + (int64_t)((r & 3) + 8 * (r >> 2)) * I1 * ZU;
        if constexpr (VEC == 1) {
          *reinterpret_cast<float2*>(o) = make_float2(z[0][r], z[1][r]);
        } else {
          *reinterpret_cast<float4*>(o) = make_float4(z[0][r], z[1][r], z[2][r], z[3][r]);
        }
      }
    }
  }
}

// -------------------------------------------------------------------------------------------
// Shared by the two last-mode kernels.  The tensor seen as (A rows, L complex per row) is cut
// into flat tiles of 32 rows (one matrix-core tile); tile t holds elements [32 t L, 32 (t + 1) L).
// `tile_start[t]` = number of support entries below 32 t L (Omega is ascending), so tile t owns
// Omega[tile_start[t] .. tile_start[t + 1]).
//
// A tile belongs to ONE wavefront from its first load to its last store, and the LDS slice it
// is staged in is private to that wavefront.  The wavefronts of a workgroup therefore never
// meet at a barrier after the factor table is staged: each runs its own load / matrix-core /
// store pipeline and the hardware overlaps them.  Workgroups have 4 wavefronts because a
// workgroup's wavefronts are spread over the 4 SIMDs of a compute unit starting at the first
// one: smaller workgroups leave the matrix cores of the last SIMDs idle.
constexpr int kTileRows = 32;

// Orders the LDS accesses of one wavefront across its lanes (LDS executes a wavefront's
// instructions in order; this only keeps the compiler from moving them across the point).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Zero in a vector register that the compiler can neither fold nor prove uniform: an index built
// with it is loaded per lane (vector memory), not through the scalar cache.
__device__ __forceinline__ int opaque_zero() {
  int z = 0;
  asm volatile("" : "+v"(z));
  return z;
}

// Factor table in LDS: sF[k * ld + m] = scale * F[m, k] as (fr, fi), ld = 16 NT, zero for k >= K
// or m >= M.  PROJECT: F[m, k] = conj(U[k, m]); otherwise F[m, k] = U[m, k].
template <bool PROJECT>
__device__ __forceinline__ void stage_factor_table(float2* sF, const float2* __restrict__ U, int rn, int K,
                                                   int M, int krows, int ld, int tid, int nthreads,
                                                   float scale = 1.f) {
  for (int e = tid; e < krows * ld; e += nthreads) {
    const int k = e / ld, m = e - k * ld;
    float2 f = make_float2(0.f, 0.f);
    if (k < K && m < M) {
      if (PROJECT) {
        const float2 u = U[(int64_t)k * rn + m];
        f = make_float2(u.x, -u.y);
      } else {
        f = U[(int64_t)m * rn + k];
      }
    }
    sF[e] = make_float2(scale * f.x, scale * f.y);
  }
}
// Coefficients of the (re, im) parts of input element k for real output column (m, p):
// re(F x) = fr xr - fi xi,  im(F x) = fi xr + fr xi.
__device__ __forceinline__ float2 column_coef(float2 f, int p) {
  return p ? make_float2(f.y, f.x) : make_float2(f.x, -f.y);
}

// Two consecutive gradient elements as they lie in memory (complex64: 16 bytes, bf16 pairs: 8).
template <int DT> struct RawPair;
template <> struct RawPair<TGRAD_C64> { typedef float4 type; };
template <> struct RawPair<TGRAD_CBF16> { typedef uint2 type; };

// Streaming accesses.  G is read once per step and W is read and written once per step; marked
// non-temporal they neither push the small reused operands (factor tables, intermediate tensors) out
// of the caches nor leave a cache full of dirty lines behind for the next kernel to wait on.
typedef float f32x4nt __attribute__((ext_vector_type(4)));
typedef float f32x2nt __attribute__((ext_vector_type(2)));
template <typename R>
__device__ __forceinline__ R nt_load(const R* p) {
  if constexpr (sizeof(R) == 16)
    return __builtin_bit_cast(R, __builtin_nontemporal_load(reinterpret_cast<const f32x4nt*>(p)));
  else
    return __builtin_bit_cast(R, __builtin_nontemporal_load(reinterpret_cast<const f32x2nt*>(p)));
}
template <typename R>
__device__ __forceinline__ void nt_store(R* p, const R& v) {
  static_assert(sizeof(R) == 16, "16-byte pieces");
  __builtin_nontemporal_store(__builtin_bit_cast(f32x4nt, v), reinterpret_cast<f32x4nt*>(p));
}

template <int DT>
__device__ __forceinline__ typename RawPair<DT>::type load_raw_pair(const void* g, int64_t p) {
  return nt_load(reinterpret_cast<const typename RawPair<DT>::type*>(g) + p);
}
template <int DT>
__device__ __forceinline__ void decode_raw(const typename RawPair<DT>::type& raw, float2& e0, float2& e1) {
  if constexpr (DT == TGRAD_C64) {
    e0 = make_float2(raw.x, raw.y);
    e1 = make_float2(raw.z, raw.w);
  } else {                                   // a bf16 is the upper half of a float32: widening is exact
    e0 = make_float2(__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xFFFF0000u));
    e1 = make_float2(__uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xFFFF0000u));
  }
}

__device__ __forceinline__ void claim_raw(float4& r) {
  asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w));
}
__device__ __forceinline__ void claim_raw(uint2& r) { asm volatile("" : "+v"(r.x), "+v"(r.y)); }

constexpr int kTileBatch = 17;            // 2-element pieces per lane in flight while a tile is staged (the most;
                                          // narrower last modes use 9 or 5: a tile of K-wide rows has K / 4 per lane)
constexpr int kJUnroll = 4;               // row pairs whose LDS operands are fetched ahead of their MFMAs
constexpr int kCoefPairs = 33;            // fused first stage: most row pairs whose coefficients stay in registers
constexpr int kCoefPairsShort = 17;       // ... and the variant for short last modes (I_N <= 34)

// k_lproj: out[a, m] = sum_k conj(U[k, m]) (G - Sparse(G, Omega))[a, k];  gs[j] = G[Omega_j].
// Wavefront w of workgroup b walks tiles b W + w, + gridDim.x W, ...; the global loads of its next
// tile are issued before the matrix-core phase of the current one.
// Matrix-core step (j, part): lanes 0..31 feed element k = 2 j, lanes 32..63 element k = 2 j + 1
// of their row (part = re, then im).  The loops carry no guards (a guarded, branchy loop ran the
// matrix cores at less than half their rate): for odd K the last pair reads element k = K of the
// row, whose coefficients are zero and whose LDS slot always holds a finite value.
//
// FUSE: the next compression stage (mode N-1, extent 32 S, rank M2 <= 32) runs on the matrix-core
// result while it is still in registers.  A wavefront then walks whole slabs (the S consecutive
// tiles that share all leading indices): the 32 x 32 result tile of stage one is, as it lies in the
// accumulator registers, the B operand of  D2[m2, (m3, p)] += F2[m2, i2] Y[i2, (m3, p)]  (register r
// holds rows d_row(r, 0) / d_row(r, 1) of the tile in the two lane halves = one row pair); the
// re/im swap of Y for the imaginary part of F2 is a swap of neighbouring lanes (DPP).  D2 is
// stored once per slab; the intermediate tensor between the two stages never exists.
struct FusedNext {
  const float2* fpad;   // conj(U^(N-1)[i2, m2]) as (re, im), zero for m2 >= M2, in operand order (k_pack_fused_factor)
  float* out;           // (slabs, M2, M) complex, row-major
  int S;                // tiles per slab; 1 when nothing is fused
  int M2;
};

template <int DT, int W, int NTB, bool FLAT, bool FUSE, int CP, int TB>
__global__ __launch_bounds__(64 * W, 2) void k_lproj(const void* __restrict__ g,
                                                     const int32_t* __restrict__ omega,
                                                     const uint32_t* __restrict__ tile_start,
                                                     float2* __restrict__ gs, const float2* __restrict__ U,
                                                     int rn, int64_t A, int K, int M, uint32_t magicK,
                                                     int64_t ntiles, float* __restrict__ out,
                                                     FusedNext fz) {
  typedef typename RawPair<DT>::type Raw;
  constexpr int T = 64 * W;
  extern __shared__ float smem[];
  constexpr bool flat = FLAT;                                  // odd K: the LDS image is the memory image
  const int stride = 2 * K + (flat ? 0 : 2);                   // floats per LDS row; stride / 2 is odd
  const int slice = kTileRows * stride + 2;                    // floats per wavefront (even)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: tile bookkeeping stays scalar
  float* sX = smem + wave * slice;
  float2* sF = reinterpret_cast<float2*>(smem + W * slice);
  const int J = (K + 1) >> 1;
  const int N2 = 2 * M;
  const int NT = (N2 + 31) >> 5;
  const int ld = 16 * NT;
  for (int e = lane; e < slice; e += 64) sX[e] = 0.f;          // pads and never-staged rows stay finite
  stage_factor_table<true>(sF, U, rn, K, M, 2 * J, ld, tid, T);
  __syncthreads();                                             // the only workgroup barrier
  // FUSE (one column tile, J <= CP): the lane's first-stage coefficients - one (re, im) pair per
  // row pair - do not depend on the tile, so they live in registers for the whole kernel and the
  // matrix-core loop reads only its A operand from LDS.  Row pairs past J carry zeros.
  float2 creg[FUSE ? CP : 1];
  if constexpr (FUSE) {
    const int c0 = lane & 31, h0 = lane >> 5;
    const float2* fl0 = sF + h0 * ld + (c0 >> 1);
#pragma unroll
    for (int j = 0; j < CP; ++j)
      creg[j] = j < J ? column_coef(fl0[2 * j * ld], c0 & 1) : make_float2(0.f, 0.f);
  }

  const int64_t I = A * K;
  const int tile_elems = kTileRows * K;
  // Tile sequence of this wavefront: slabs wg, wg + nw, ... and inside a slab its S tiles in order
  // (S = 1 without fusion, where a slab is a tile).
  const int S = FUSE ? fz.S : 1;
  const int64_t nslabs = (ntiles + S - 1) / S;
  const int64_t nw = (int64_t)gridDim.x * W;
  int64_t slab = (int64_t)blockIdx.x * W + wave;
  int ts = 0;
  if (slab >= nslabs) return;
  auto advance = [&](int64_t& sl, int& t) {                    // next position of the sequence
    if (t + 1 < S) { t += 1; } else { t = 0; sl += nw; }
  };

  Raw raw[TB];
  int32_t my_om = -1;
  // issue the first batch of tile `t` (its support range is [j0, j1)) into raw / my_om.  The loads
  // are unconditional (indices past the tile are clamped onto its last pair): a conditional load
  // would be followed by a wait and a register copy.
  auto issue = [&](int64_t t, uint32_t j0, uint32_t j1) {
    const int64_t e_base = t * tile_elems;
    const int n_e = (int)((I - e_base) < tile_elems ? (I - e_base) : tile_elems);
    const int npairs = n_e >> 1;                               // >= 1: the host keeps K >= 2 here
#pragma unroll
    for (int i = 0; i < TB; ++i) {
      const int pi = lane + i * 64;
      raw[i] = load_raw_pair<DT>(g, (e_base >> 1) + (pi < npairs ? pi : npairs - 1));
    }
    my_om = (j0 + lane < j1) ? omega[j0 + lane] : -1;
  };
  // element pair at flat offset e0 of the tile -> LDS
  auto commit_pair = [&](const Raw& rw, int e0) {
    float2 v0, v1;
    decode_raw<DT>(rw, v0, v1);
    if (flat) {
      *reinterpret_cast<float4*>(&sX[2 * e0]) = make_float4(v0.x, v0.y, v1.x, v1.y);
    } else {
      const uint32_t r0 = div_magic((uint32_t)e0, magicK);
      const uint32_t c0 = (uint32_t)e0 - r0 * (uint32_t)K;
      const bool wrap = c0 + 1 == (uint32_t)K;
      const uint32_t r1 = wrap ? r0 + 1 : r0;
      const uint32_t c1 = wrap ? 0u : c0 + 1;
      *reinterpret_cast<float2*>(&sX[r0 * stride + 2 * c0]) = v0;
      *reinterpret_cast<float2*>(&sX[r1 * stride + 2 * c1]) = v1;
    }
  };

  // The support ranges are fetched with per-lane (vector) loads on purpose: a scalar load shares
  // its wait counter with the LDS reads of the matrix-core phase and would stall its first step.
  const int vzero = opaque_zero();
  int64_t tile = slab * S;
  int64_t nslab = slab;
  int nts = ts;
  advance(nslab, nts);
  bool have_next = nslab < nslabs;
  int64_t nxt = have_next ? nslab * S + nts : tile;            // past the end: reload the current tile (unused)
  uint32_t cj0 = tile_start[tile + vzero], cj1 = tile_start[tile + 1 + vzero];
  uint32_t nj0 = tile_start[nxt + vzero], nj1 = tile_start[nxt + 1 + vzero];
  issue(tile, cj0, cj1);
  v16f acc2;                                                   // FUSE: second-stage accumulator of the slab
#pragma unroll
  for (int r = 0; r < 16; ++r) acc2[r] = 0.f;
  while (true) {
    const int64_t e_base = tile * tile_elems;
    const int n_e = (int)((I - e_base) < tile_elems ? (I - e_base) : tile_elems);
    wave_sync();                                               // previous tile's LDS reads are done
    // Opaque copy of the lane id: everything addressed through it is recomputed per tile (a few
    // VALU operations) instead of being hoisted into dozens of long-lived registers, which
    // would spill - and a spill reload waits for every load in flight.
    int lane_now = lane;
    asm volatile("" : "+v"(lane_now));
    const int col = lane_now & 31, half = lane_now >> 5;
    const float* xa = sX + col * stride + 2 * half;            // the lane's own row, its half of each pair
    const float2* fl = sF + half * ld + (col >> 1);
    const int part = col & 1;
    // one wait for the whole batch (the only memory operations issued after it were loads)
    asm volatile("" : "+v"(my_om));
#pragma unroll
    for (int i = 0; i < TB; ++i) claim_raw(raw[i]);
    const int npairs = n_e >> 1;
#pragma unroll
    for (int i = 0; i < TB; ++i) {
      const int pi = lane_now + i * 64;
      if (pi < npairs) commit_pair(raw[i], 2 * pi);
    }
    for (int pi = lane + TB * 64; pi < npairs; pi += 64)          // long rows: the rest, unpipelined
      commit_pair(load_raw_pair<DT>(g, (e_base >> 1) + pi), 2 * pi);
    if ((n_e & 1) && lane == 0) {                              // odd element count: the last one alone
      const int e = n_e - 1;
      const float2 v = load_elem<DT>(g, e_base + e);
      const uint32_t r = div_magic((uint32_t)e, magicK);
      *reinterpret_cast<float2*>(&sX[r * stride + 2 * ((uint32_t)e - r * (uint32_t)K)]) = v;
    }
    // ---- second-stage factor operands of this tile (FUSE): small, cache-resident; issued before
    //      the next tile's loads so that waiting for them leaves those in flight ----
    float2 f2s[FUSE ? 16 : 1];
    if constexpr (FUSE) {
      const float4* fp = reinterpret_cast<const float4*>(fz.fpad) + (size_t)ts * 8 * 64 + lane_now;
#pragma unroll
      for (int rp = 0; rp < 8; ++rp) {
        const float4 f = fp[rp * 64];
        f2s[2 * rp] = make_float2(f.x, f.y);
        f2s[2 * rp + 1] = make_float2(f.z, f.w);
      }
    }
    // ---- the staging registers are free: the next tile's loads go in flight right away (its
    //      support range was fetched one tile earlier).  All unconditional: see `issue`. ----
    const int32_t cur_om = my_om;
    int64_t nnslab = nslab;
    int nnts = nts;
    advance(nnslab, nnts);
    const bool have_nn = have_next && nnslab < nslabs;
    const int64_t nn = have_nn ? nnslab * S + nnts : nxt;
    issue(nxt, nj0, nj1);
    const uint32_t nnj0 = tile_start[nn + vzero], nnj1 = tile_start[nn + 1 + vzero];
    wave_sync();
    // ---- Sparse(G, Omega) of this tile: hand the values over, then remove them ----
    // (the first 64 entries of the tile were prefetched with it: the common path loads nothing, so
    // it never waits for the loads just issued; longer ranges take the rare second loop)
    auto take_entry = [&](uint32_t j, int32_t oj) {
      const uint32_t e = (uint32_t)((int64_t)oj - e_base);
      const uint32_t r = flat ? 0u : div_magic(e, magicK);
      float2* p = reinterpret_cast<float2*>(&sX[r * stride + 2 * (e - r * (uint32_t)K)]);
      gs[j] = *p;
      *p = make_float2(0.f, 0.f);
    };
    if (cj0 + lane < cj1) take_entry(cj0 + lane, cur_om);
    if (cj1 - cj0 > 64u)
      for (uint32_t j = cj0 + 64u + lane; j < cj1; j += 64) take_entry(j, omega[j]);
    wave_sync();
    // ---- the 32 rows through the matrix cores, NTB column tiles at a time ----
    const int64_t grow0 = tile * kTileRows;
    auto block = [&](int nt0, auto ntile_count) {
      constexpr int N = decltype(ntile_count)::value;
      v16f acc[N];
#pragma unroll
      for (int i = 0; i < N; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
      const float2* fb = fl + 16 * nt0;
      int j = 0;
      if constexpr (FUSE) {
        // straight-line: CP row pairs, A operands fetched kJUnroll pairs ahead; pairs past J re-read
        // the last one and meet zero coefficients
        const int jlast = J - 1;
        float2 a2[kJUnroll];
#pragma unroll
        for (int u = 0; u < kJUnroll; ++u) a2[u] = *reinterpret_cast<const float2*>(xa + 4 * (u < jlast ? u : jlast));
#pragma unroll
        for (int jj = 0; jj < CP; ++jj) {
          const float2 a = a2[jj % kJUnroll];
          if (jj + kJUnroll < CP) {
            const int jn = jj + kJUnroll;
            a2[jj % kJUnroll] = *reinterpret_cast<const float2*>(xa + 4 * (jn < jlast ? jn : jlast));
          }
          acc[0] = mfma32(a.x, creg[jj].x, acc[0]);
          acc[0] = mfma32(a.y, creg[jj].y, acc[0]);
        }
        j = J;
      }
      for (; j + kJUnroll <= J; j += kJUnroll) {
        float2 a2[kJUnroll], f2[kJUnroll][N];
#pragma unroll
        for (int u = 0; u < kJUnroll; ++u) {
          a2[u] = *reinterpret_cast<const float2*>(xa + 4 * (j + u));
#pragma unroll
          for (int i = 0; i < N; ++i) f2[u][i] = fb[2 * (j + u) * ld + 16 * i];
        }
#pragma unroll
        for (int u = 0; u < kJUnroll; ++u)
#pragma unroll
          for (int i = 0; i < N; ++i) {
            const float2 b2 = column_coef(f2[u][i], part);
            acc[i] = mfma32(a2[u].x, b2.x, acc[i]);
            acc[i] = mfma32(a2[u].y, b2.y, acc[i]);
          }
      }
      for (; j < J; ++j) {
        const float2 a2 = *reinterpret_cast<const float2*>(xa + 4 * j);
#pragma unroll
        for (int i = 0; i < N; ++i) {
          const float2 b2 = column_coef(fb[2 * j * ld + 16 * i], part);
          acc[i] = mfma32(a2.x, b2.x, acc[i]);
          acc[i] = mfma32(a2.y, b2.y, acc[i]);
        }
      }
      if constexpr (FUSE) {                                    // NT == 1, N == 1
        asm volatile("" : "+v"(f2s[0].x));                     // the factor operands are claimed here
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float y = acc[0][r];
          const float sw = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(y), 0xB1, 0xF, 0xF, true));
          const float yj = part ? sw : -sw;                    // (Y J): re column <- -im, im column <- re
          acc2 = mfma32(f2s[r].x, y, acc2);
          acc2 = mfma32(f2s[r].y, yj, acc2);
        }
        if (ts == S - 1) {                                     // slab complete: D2 -> out[slab, m2, c]
          float* o = fz.out + (size_t)slab * fz.M2 * N2 + col;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int m2 = d_row(r, half);
            if (m2 < fz.M2 && col < N2) o[m2 * N2] = acc2[r];
            acc2[r] = 0.f;
          }
        }
      } else {
#pragma unroll
        for (int i = 0; i < N; ++i) {
          const int c = 32 * (nt0 + i) + col;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int64_t grow = grow0 + d_row(r, half);
            if (grow < A && c < N2) out[grow * N2 + c] = acc[i][r];
          }
        }
      }
    };
    if constexpr (FUSE) {
      __builtin_amdgcn_s_setprio(1);                           // matrix-core phase: ahead of the other wavefront's loads and stores
      block(0, std::integral_constant<int, 1>());              // exactly one column tile (and no loop around the
    } else {                                                   // claim of f2s: a loop preheader would drain all loads)
      int nt0 = 0;
      for (; nt0 + NTB <= NT; nt0 += NTB) block(nt0, std::integral_constant<int, NTB>());
      if (NTB > 1)
        for (; nt0 < NT; ++nt0) block(nt0, std::integral_constant<int, 1>());
    }
    if constexpr (FUSE) __builtin_amdgcn_s_setprio(0);
    if (!have_next) break;
    tile = nxt;
    slab = nslab;
    ts = nts;
    nxt = nn;
    nslab = nnslab;
    nts = nnts;
    have_next = have_nn;
    cj0 = nj0;
    cj1 = nj1;
    nj0 = nnj0;
    nj1 = nnj1;
  }
}

// -------------------------------------------------------------------------------------------
// k_lproj_flat: k_lproj<.., FUSE> for odd last extents (the LDS image of a tile is its memory image),
// written so that everything a wavefront does OUTSIDE its matrix-core phase is scalar, LDS or
// vector-memory work with loop-invariant vector registers.  fp32 MFMA instructions run on the SIMD's
// vector ALU: while one wavefront of a SIMD is in its matrix-core phase, a vector-ALU instruction of
// the other one does not issue, so address arithmetic, clamps and lane masks in the staging phase
// serialise the two wavefronts instead of overlapping them.  Here
//  - the tile is fetched with buffer loads: the descriptor (scalar registers) carries the tile's
//    base and size, lanes past the tile's end read zero without touching memory, and the lane's
//    offset is one invariant register;
//  - every lane commits what it loaded (the slice has room for TB x 64 pieces; the host picks TB so
//    that they cover the tile: TB x 64 >= 16 K), so no lane masks;
//  - support ranges, factor operands and results go through scalar bases + invariant lane offsets.
// Same tile sequence and the same arithmetic, in the same order, as k_lproj<.., FUSE>.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_buffer(const void* base, uint32_t bytes) {
  // untyped buffer, stride 0: an access at offset >= bytes returns zero (loads) or is dropped (stores)
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), (short)0, (int)bytes, 0x00020000);
}
// Two consecutive gradient elements as a buffer load returns them (one register tuple), and their
// float32 image in LDS.
template <int DT> struct BufPair;
template <> struct BufPair<TGRAD_C64> {
  typedef u32x4 type;
  static __device__ __forceinline__ type load(__amdgpu_buffer_rsrc_t r, int voff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0, 2);   // cache policy: non-temporal
  }
  static __device__ __forceinline__ void commit(float* dst, const type& v) { *reinterpret_cast<type*>(dst) = v; }
};
template <> struct BufPair<TGRAD_CBF16> {
  typedef u32x2 type;
  static __device__ __forceinline__ type load(__amdgpu_buffer_rsrc_t r, int voff) {
    return __builtin_amdgcn_raw_buffer_load_b64(r, voff, 0, 2);    // cache policy: non-temporal
  }
  static __device__ __forceinline__ void commit(float* dst, const type& v) {   // a bf16 is the upper half of a float32
    u32x4 w;
    w.x = v.x << 16;
    w.y = v.x & 0xFFFF0000u;
    w.z = v.y << 16;
    w.w = v.y & 0xFFFF0000u;
    *reinterpret_cast<u32x4*>(dst) = w;
  }
};

// floats of LDS per wavefront: the tile (32 rows of K complex + one pad pair for the row pair past
// an odd K) or, if larger, what TB x 64 committed pieces cover; a multiple of 4 (16-byte writes)
__host__ __device__ inline int lproj_flat_slice(int K, int TB) {
  const int tile = kTileRows * 2 * K + 2, staged = TB * 64 * 4;
  return ((tile > staged ? tile : staged) + 3) & ~3;
}

template <int DT, int CP, int TB>
__global__ __launch_bounds__(256, 2) void k_lproj_flat(const void* __restrict__ g,
                                                       const int32_t* __restrict__ omega,
                                                       const uint32_t* __restrict__ tile_start,
                                                       float2* __restrict__ gs, const float2* __restrict__ U,
                                                       int rn, int64_t A, int K, int M, int64_t ntiles,
                                                       FusedNext fz) {
  typedef typename BufPair<DT>::type Raw;
  constexpr int W = 4, T = 64 * W;
  constexpr int kPiece = (int)sizeof(Raw);                     // bytes of G per lane and load (2 elements)
  constexpr int kLoadEvery = (CP - 1) / (TB - 1) >= 2 ? 2 : 1; // row pairs of the first stage per load of the next tile
  static_assert((TB - 1) * kLoadEvery < CP, "the first stage issues all TB loads");
  extern __shared__ float smem[];
  const int stride = 2 * K;                                    // floats per LDS row; K is odd
  const int slice = lproj_flat_slice(K, TB);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  float* sX = smem + wave * slice;
  float2* sF = reinterpret_cast<float2*>(smem + W * slice);
  const int J = (K + 1) >> 1;
  const int N2 = 2 * M;                                        // <= 32: one column tile
  const int ld = 16;
  for (int e = lane; e < slice; e += 64) sX[e] = 0.f;          // pads stay finite
  stage_factor_table<true>(sF, U, rn, K, M, 2 * J, ld, tid, T);
  __syncthreads();                                             // the only workgroup barrier
  const int col = lane & 31, half = lane >> 5, part = col & 1;
  float2 creg[CP];                                             // first-stage coefficients, one pair per row pair
  {
    const float2* fl0 = sF + half * ld + (col >> 1);
#pragma unroll
    for (int j = 0; j < CP; ++j)
      creg[j] = j < J ? column_coef(fl0[2 * j * ld], part) : make_float2(0.f, 0.f);
  }
  float sgn = part ? 1.f : -1.f;                               // (Y J): re column <- -im, im column <- re
  asm volatile("" : "+v"(sgn));                                // (kept a multiplication: it takes the lane swap as its operand modifier)

  const uint32_t tile_elems = (uint32_t)(kTileRows * K);
  const uint32_t tile_bytes = tile_elems * (uint32_t)(kPiece / 2);
  const int S = fz.S;
  const int nslabs = (int)(ntiles / S);                        // whole slabs (host); tile counts fit 32 bits
  const int nw = (int)gridDim.x * W;
  int slab = (int)blockIdx.x * W + wave;
  int ts = 0;
  if (slab >= nslabs) return;
  auto advance = [&](int& sl, int& t) {
    if (t + 1 < S) { t += 1; } else { t = 0; sl += nw; }
  };
  // loop-invariant lane addresses
  const int voff_g = lane * kPiece;                            // into the tile, bytes
  float* sW = sX + lane * 4;                                   // commit: piece i goes to sW + i * 256
  const float* xa = sX + col * stride + 2 * half;              // matrix-core A operand: own row, own half of a pair
  const bool full_out = fz.M2 == 32 && N2 == 32;
  const uint32_t voff_out = (uint32_t)(4 * half * N2 + col);

  Raw raw[TB];
  int32_t my_om = 0;
  // bytes of the tile from the first piece of every group of 4 loads on (scalar registers: a
  // saturating subtraction inside the loop would be done by the vector ALU)
  constexpr int kGroups = (TB + 3) / 4;
  uint32_t rest[kGroups];
#pragma unroll
  for (int k = 0; k < kGroups; ++k) {
    const uint32_t done = (uint32_t)(k * 4 * 64 * kPiece);
    rest[k] = __builtin_amdgcn_readfirstlane(tile_bytes > done ? tile_bytes - done : 0u);
  }
  // piece i of tile t -> raw[i]; the first 64 support entries of a tile -> my_om.  Nothing here uses
  // the vector ALU.  (A descriptor per 4 pieces: immediate offsets reach 4 KB.)
  auto issue_piece = [&](int t, int i) {
    const char* tb = reinterpret_cast<const char*>(g) + (int64_t)t * (int64_t)tile_bytes;
    const int k = i / 4;
    const __amdgpu_buffer_rsrc_t r = raw_buffer(tb + (uint32_t)(k * 4 * 64 * kPiece), rest[k]);
    raw[i] = BufPair<DT>::load(r, voff_g + (i - 4 * k) * 64 * kPiece);
  };
  auto issue_support = [&](uint32_t j0, uint32_t j1) {
    const uint32_t cnt = j1 - j0;                              // (s_min_u32: scalar)
    const __amdgpu_buffer_rsrc_t ro = raw_buffer(omega + j0, (cnt < 64u ? cnt : 64u) * 4u);
    my_om = (int32_t)__builtin_amdgcn_raw_buffer_load_b32(ro, lane * 4, 0, 0);
  };
  const uint32_t vzero = (uint32_t)opaque_zero();
  auto range_of = [&](int t, uint32_t& j0, uint32_t& j1) {   // per-lane loads (scalar base), made scalar when used
    const uint32_t* tsb = tile_start + t;
    j0 = tsb[vzero];
    j1 = tsb[vzero + 1];
  };
  int tile = slab * S;
  int nslab = slab;
  int nts = ts;
  advance(nslab, nts);
  bool have_next = nslab < nslabs;
  int nxt = have_next ? nslab * S + nts : tile;            // past the end: reload the current tile (unused)
  uint32_t cj0v, cj1v, nj0v, nj1v;
  range_of(tile, cj0v, cj1v);
  range_of(nxt, nj0v, nj1v);
  uint32_t cj0 = __builtin_amdgcn_readfirstlane(cj0v), cj1 = __builtin_amdgcn_readfirstlane(cj1v);
#pragma unroll
  for (int i = 0; i < TB; ++i) issue_piece(tile, i);
  issue_support(cj0, cj1);
  v16f acc2;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc2[r] = 0.f;
  // D2 of a complete slab -> out[slab, m2, c].  Issued at the start of the NEXT tile's staging phase,
  // not after the last matrix-core instruction: the wait that opens a tile covers every vector-memory
  // operation before it, and stores issued just before it would be waited for in full.
  auto store_slab = [&](int sl) {
    float* ob = fz.out + (size_t)sl * fz.M2 * N2;
    if (full_out) {                                            // scalar row bases + one invariant lane offset
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float* orow = ob + ((r & 3) + 8 * (r >> 2)) * N2;
        orow[voff_out] = acc2[r];
        acc2[r] = 0.f;
      }
    } else {                                                   // narrower ranks: guarded, addresses made on the spot
      int lane_now = lane;                                     // (opaque: nothing of this is kept in registers across tiles)
      asm volatile("" : "+v"(lane_now));
      const int c2 = lane_now & 31, h2 = lane_now >> 5;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m2 = d_row(r, h2);
        if (m2 < fz.M2 && c2 < N2) ob[m2 * N2 + c2] = acc2[r];
        acc2[r] = 0.f;
      }
    }
  };
  bool pending = false;
  int pending_slab = 0;
  while (true) {
    const uint32_t e_base = (uint32_t)tile * tile_elems;        // I < 2^31
    wave_sync();                                               // previous tile's LDS reads are done
    asm volatile("" : "+v"(my_om));
#pragma unroll
    for (int i = 0; i < TB; ++i) asm volatile("" : "+v"(raw[i]));   // one wait for the whole batch
#pragma unroll
    for (int i = 0; i < TB; ++i) BufPair<DT>::commit(sW + i * 256, raw[i]);
    __builtin_amdgcn_sched_barrier(0);                         // (loads moved above these writes would need register copies)
    if (pending) store_slab(pending_slab);
    // second-stage factor operands of this tile: small, cache-resident; before the next tile's loads
    float2 f2s[16];
    {
      const float4* fp = reinterpret_cast<const float4*>(fz.fpad) + (size_t)ts * 8 * 64;
#pragma unroll
      for (int rp = 0; rp < 8; ++rp) {
        const float4 f = fp[rp * 64 + lane];
        f2s[2 * rp] = make_float2(f.x, f.y);
        f2s[2 * rp + 1] = make_float2(f.z, f.w);
      }
    }
    const int32_t cur_om = my_om;
    int nnslab = nslab;
    int nnts = nts;
    advance(nnslab, nnts);
    const bool have_nn = have_next && nnslab < nslabs;
    const int nn = have_nn ? nnslab * S + nnts : nxt;
    const uint32_t nj0 = __builtin_amdgcn_readfirstlane(nj0v), nj1 = __builtin_amdgcn_readfirstlane(nj1v);
    wave_sync();
    // Sparse(G, Omega) of this tile: hand the values over, then remove them
    {
      float2* gsb = gs + cj0;
      const uint32_t cnt = cj1 - cj0;
      if ((uint32_t)lane < cnt) {
        const uint32_t e = (uint32_t)cur_om - e_base;            // the entry lies in this tile
        float2* p = reinterpret_cast<float2*>(sX + 2 * e);
        gsb[lane] = *p;
        *p = make_float2(0.f, 0.f);
      }
      if (cnt > 64u)
        for (uint32_t j = 64u + lane; j < cnt; j += 64) {
          const uint32_t e = (uint32_t)omega[cj0 + j] - e_base;
          float2* p = reinterpret_cast<float2*>(sX + 2 * e);
          gsb[j] = *p;
          *p = make_float2(0.f, 0.f);
        }
    }
    wave_sync();
    // ---- the 32 rows through the matrix cores ----
    __builtin_amdgcn_s_setprio(1);
    v16f acc;
    {
      // CP row pairs, straight-line, A operands fetched kJUnroll pairs ahead at constant offsets.  Pairs
      // past J meet zero coefficients; what they read lies in the wavefront's own slice (the host
      // checks 62 K + 4 CP <= TB x 256) and is tile data or zeros, so it is finite.
      float2 a2[kJUnroll];
#pragma unroll
      for (int u = 0; u < kJUnroll; ++u) a2[u] = *reinterpret_cast<const float2*>(xa + 4 * u);
#pragma unroll
      for (int jj = 0; jj < CP; ++jj) {
        const float2 a = a2[jj % kJUnroll];
        if (jj + kJUnroll < CP) a2[jj % kJUnroll] = *reinterpret_cast<const float2*>(xa + 4 * (jj + kJUnroll));
        if (jj == 0) {
          v16f zero;
#pragma unroll
          for (int r = 0; r < 16; ++r) zero[r] = 0.f;
          acc = mfma32(a.x, creg[0].x, zero);
        } else {
          acc = mfma32(a.x, creg[jj].x, acc);
        }
        acc = mfma32(a.y, creg[jj].y, acc);
        // The next tile's loads, one per row pair: a load instruction waits at issue until the memory
        // pipeline takes it (at the rate memory delivers when every wavefront streams), and here that
        // wait lies under the matrix-core instructions instead of in front of them.
        if (jj % kLoadEvery == 0 && jj / kLoadEvery < TB) {
          __builtin_amdgcn_sched_barrier(0);
          issue_piece(nxt, jj / kLoadEvery);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    issue_support(nj0, nj1);
    uint32_t nnj0v, nnj1v;
    range_of(nn, nnj0v, nnj1v);
    asm volatile("" : "+v"(f2s[0].x));                         // the factor operands are claimed here
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float y = acc[r];
      const float sw = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(y), 0xB1, 0xF, 0xF, true));
      const float yj = sw * sgn;
      acc2 = mfma32(f2s[r].x, y, acc2);
      acc2 = mfma32(f2s[r].y, yj, acc2);
    }
    const bool slab_done = ts == S - 1;
    const int done_slab = slab;
    __builtin_amdgcn_s_setprio(0);
    pending = slab_done;
    pending_slab = done_slab;
    if (!have_next) break;
    tile = nxt;
    slab = nslab;
    ts = nts;
    nxt = nn;
    nslab = nnslab;
    nts = nnts;
    have_next = have_nn;
    cj0 = nj0;
    cj1 = nj1;
    nj0v = nnj0v;
    nj1v = nnj1v;
  }
  if (pending) store_slab(pending_slab);
}

// k_lupdate: tile = c_alpha * (z x_N U) + c_lambda * scatter(N_S);  W <- decay * W + tile,
// with c_alpha = -lr alpha, c_lambda = -lr lambda, decay = 1 - lr wd (Algorithm 1: "Reconstruct
// low-rank part", "Add scaled sparse tensor", weight update; AdamUpdate on the sparse values
// as in the appendix algorithm "Adam with low-rank tensor decomposition").
// The rows of z are read straight into matrix-core operand registers: lane (row, half) keeps
// elements k = half JT .. half JT + JT - 1 of its row (JT = a power of two >= K / 2, zero beyond
// K), so step (j, part) pairs element j (lanes 0..31) with element JT + j (lanes 32..63).
struct SparseAdam {
  const int32_t* omega;
  const uint32_t* tile_start;
  const float2* gs;
  float2* ms;
  float* vs;
  float beta1, beta2, inv_c1, inv_c2, eps, c_lambda;
  int k_last;           // max(k, 1) - 1: a support position that is always safe to read
};

// AdamUpdate on sparse entry j (value x at support position oj, moments mm / v_old) and
// tile[oj] += (-lr lambda) N_S[j]; `sD` is the flat LDS image of the W tile that starts at w_base.
__device__ __forceinline__ void sparse_adam_entry(const SparseAdam& sp, uint32_t j, int32_t oj, float2 x,
                                                  float2 mm, float v_old, int64_t w_base, float* sD) {
  mm.x = sp.beta1 * mm.x + (1.f - sp.beta1) * x.x;
  mm.y = sp.beta1 * mm.y + (1.f - sp.beta1) * x.y;
  const float vv = sp.beta2 * v_old + (1.f - sp.beta2) * (x.x * x.x + x.y * x.y);
  sp.ms[j] = mm;
  sp.vs[j] = vv;
  const float d = sp.c_lambda * sp.inv_c1 / (sqrtf(vv * sp.inv_c2) + sp.eps);
  const int e = (int)((int64_t)oj - w_base);
  sD[2 * e] += d * mm.x;
  sD[2 * e + 1] += d * mm.y;
}

constexpr int kUpdPrefetch = 17;          // complex64 pairs of W per lane kept in flight during the MFMA phase (the
                                          // most; narrower last modes use 9 or 5: a tile of M-wide rows has M / 4)

// float32 -> bf16 bit pattern, round to nearest, ties to even (NaN stays a quiet NaN).
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t bf16_pack(float re, float im) { return bf16_rne(re) | (bf16_rne(im) << 16); }

// How the weight tensor is stored (section "Mixed precision training": weights may be kept in half
// precision while the optimizer states stay in full precision).  A "piece" is 16 bytes of the W tile:
// 2 complex64 elements, or 4 elements stored as bf16 (re, im) pairs.  apply() returns
// decay * w + d for the piece, d read from the float32 image `sD` of the tile's update; bf16 weights
// are widened exactly, updated in float32 and rounded once (nearest even).
template <int WDT> struct WStore;
template <> struct WStore<TGRAD_C64> {
  typedef float4 raw;
  static constexpr int kElems = 2;
  static __device__ __forceinline__ raw* tile(void* w, int64_t w_base) {
    return reinterpret_cast<raw*>(reinterpret_cast<float*>(w) + 2 * w_base);
  }
  static __device__ __forceinline__ raw apply(const raw o, const float* sD, int q, float decay) {
    const float4 d = reinterpret_cast<const float4*>(sD)[q];
    return make_float4(decay * o.x + d.x, decay * o.y + d.y, decay * o.z + d.z, decay * o.w + d.w);
  }
  static __device__ __forceinline__ void apply_one(void* w, int64_t e, const float* d, float decay) {
    float2* p = reinterpret_cast<float2*>(w) + e;
    const float2 o = *p;
    *p = make_float2(decay * o.x + d[0], decay * o.y + d[1]);
  }
};
template <> struct WStore<TGRAD_CBF16> {
  typedef uint4 raw;
  static constexpr int kElems = 4;
  static __device__ __forceinline__ raw* tile(void* w, int64_t w_base) {
    return reinterpret_cast<raw*>(reinterpret_cast<uint32_t*>(w) + w_base);
  }
  static __device__ __forceinline__ uint32_t one(uint32_t o, float dre, float dim, float decay) {
    return bf16_pack(decay * __uint_as_float(o << 16) + dre, decay * __uint_as_float(o & 0xFFFF0000u) + dim);
  }
  static __device__ __forceinline__ raw apply(const raw o, const float* sD, int q, float decay) {
    const float4 d0 = reinterpret_cast<const float4*>(sD)[2 * q];
    const float4 d1 = reinterpret_cast<const float4*>(sD)[2 * q + 1];
    return make_uint4(one(o.x, d0.x, d0.y, decay), one(o.y, d0.z, d0.w, decay), one(o.z, d1.x, d1.y, decay),
                      one(o.w, d1.z, d1.w, decay));
  }
  static __device__ __forceinline__ void apply_one(void* w, int64_t e, const float* d, float decay) {
    uint32_t* p = reinterpret_cast<uint32_t*>(w) + e;
    *p = one(*p, d[0], d[1], decay);
  }
};
__device__ __forceinline__ void claim_raw(uint4& r) { asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w)); }
// 16-byte pieces of W through a buffer descriptor (range-checked by the hardware: no clamps, no lane
// masks), non-temporal
__device__ __forceinline__ void buffer_piece_load(float4& d, __amdgpu_buffer_rsrc_t r, int voff) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0, 2);
  d = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
__device__ __forceinline__ void buffer_piece_load(uint4& d, __amdgpu_buffer_rsrc_t r, int voff) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0, 2);
  d = make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void buffer_piece_store(const float4& d, __amdgpu_buffer_rsrc_t r, int voff) {
  u32x4 v;
  v.x = __float_as_uint(d.x);
  v.y = __float_as_uint(d.y);
  v.z = __float_as_uint(d.z);
  v.w = __float_as_uint(d.w);
  __builtin_amdgcn_raw_buffer_store_b128(v, r, voff, 0, 2);
}
__device__ __forceinline__ void buffer_piece_store(const uint4& d, __amdgpu_buffer_rsrc_t r, int voff) {
  u32x4 v;
  v.x = d.x;
  v.y = d.y;
  v.z = d.z;
  v.w = d.w;
  __builtin_amdgcn_raw_buffer_store_b128(v, r, voff, 0, 2);
}

template <int WDT, int W, int NTB, int JT, int UP>
__global__ __launch_bounds__(64 * W, 2) void k_lupdate(const float* __restrict__ z,
                                                       const float2* __restrict__ U, int64_t A, int K,
                                                       int M, int64_t ntiles, void* __restrict__ w,
                                                       float decay, float c_alpha, SparseAdam sp) {
  typedef WStore<WDT> WS;
  typedef typename WS::raw wraw;
  constexpr int kPre = WS::kElems == 2 ? UP : (UP + 1) / 2;   // 16-byte pieces of the W tile per lane in flight
  constexpr int T = 64 * W;
  extern __shared__ float smem[];
  const int N2 = 2 * M;
  const int NT = (N2 + 31) >> 5;
  const int ld = 16 * NT;
  const int slice = (kTileRows * N2 + 3) & ~3;                 // floats per wavefront: flat image of its W tile
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: tile bookkeeping stays scalar
  float* sD = smem + wave * slice;
  float2* sF = reinterpret_cast<float2*>(smem + W * slice);
  stage_factor_table<false>(sF, U, K, K, M, 2 * JT, ld, tid, T, c_alpha);   // the update's scale rides in the table
  __syncthreads();                                             // the only workgroup barrier
  // a lone last complex column (half-spectrum modes have 2^m + 1 entries) does not get a 32-column
  // matrix-core tile of its own: it is expanded with vector arithmetic (see k_lupdate_fused)
  const bool vtail = (N2 & 31) == 2;
  const int NTm = vtail ? NT - 1 : NT;

  const int64_t Iw = A * M;                                    // complex elements of W
  const int tile_w = kTileRows * M;
  const int64_t step = (int64_t)gridDim.x * W;
  int64_t tile = (int64_t)blockIdx.x * W + wave;
  if (tile >= ntiles) return;
  const float2* zall = reinterpret_cast<const float2*>(z);

  float2 zreg[JT];
  int32_t my_om = -1;
  float2 my_g = make_float2(0.f, 0.f), my_m = make_float2(0.f, 0.f);
  float my_v = 0.f;
  // operand rows and sparse state of tile `t` (support range [j0, j1))
  auto issue_small = [&](int64_t t, uint32_t j0, uint32_t j1) {
    const int col = lane & 31, half = lane >> 5;
    const int64_t grow = t * kTileRows + col;
    const float2* zr = zall + grow * K + half * JT;
#pragma unroll
    for (int j = 0; j < JT; ++j) {
      zreg[j] = make_float2(0.f, 0.f);
      if (grow < A && half * JT + j < K) zreg[j] = zr[j];
    }
    my_om = -1;
    if (j0 + lane < j1) {
      my_om = sp.omega[j0 + lane];
      my_g = sp.gs[j0 + lane];
      my_m = sp.ms[j0 + lane];
      my_v = sp.vs[j0 + lane];
    }
  };

  const int vzero = opaque_zero();                             // see k_lproj
  int64_t nxt = tile + step;
  uint32_t cj0 = sp.tile_start[tile + vzero], cj1 = sp.tile_start[tile + 1 + vzero];
  uint32_t nj0 = 0, nj1 = 0;
  if (nxt < ntiles) {
    nj0 = sp.tile_start[nxt + vzero];
    nj1 = sp.tile_start[nxt + 1 + vzero];
  }
  // Every wait for loads sits at ONE point per tile (claim_loads, before the stream-out), where the
  // only younger memory operations are loads that are needed right after anyway.  Loads retire
  // in order, so a wait anywhere else would also wait for stores or loads issued after it.
  auto claim_small = [&]() {
#pragma unroll
    for (int j = 0; j < JT; ++j) asm volatile("" : "+v"(zreg[j].x), "+v"(zreg[j].y));
    asm volatile("" : "+v"(my_om), "+v"(my_g.x), "+v"(my_g.y), "+v"(my_m.x), "+v"(my_m.y), "+v"(my_v));
  };
  issue_small(tile, cj0, cj1);
  claim_small();
  while (true) {
    int lane_now = lane;                                       // opaque per-tile copy (see k_lproj)
    asm volatile("" : "+v"(lane_now));
    const int col = lane_now & 31, half = lane_now >> 5;
    const float2* fl = sF + half * JT * ld + (col >> 1);
    const int part = col & 1;
    const int64_t w_base = tile * tile_w;                      // complex index of the tile in W
    const int n_w = (int)((Iw - w_base) < tile_w ? (Iw - w_base) : tile_w);
    wraw* w4 = WS::tile(w, w_base);                            // 16-byte aligned: a tile holds 32 M elements
    const int n4 = n_w / WS::kElems;                           // whole 16-byte pieces
    // ---- what was fetched one tile ago moves out of the prefetch registers; the next tile's small
    //      loads and this tile's W pieces go in flight ----
    float2 zcur[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j) zcur[j] = zreg[j];
    const int32_t c_om = my_om;
    const float2 c_g = my_g, c_m = my_m;
    const float c_v = my_v;
    const int64_t nn = nxt + step;
    uint32_t nnj0 = 0, nnj1 = 0;
    if (nxt < ntiles) {
      issue_small(nxt, nj0, nj1);
      if (nn < ntiles) {
        nnj0 = sp.tile_start[nn + vzero];
        nnj1 = sp.tile_start[nn + 1 + vzero];
      }
    }
    wraw wpre[kPre];                                  // unconditional loads, clamped onto the last
#pragma unroll                                                 // piece (the host keeps n4 >= 1 for every tile)
    for (int i = 0; i < kPre; ++i) {
      const int q = lane_now + i * 64;
      wpre[i] = nt_load(&w4[q < n4 ? q : n4 - 1]);
    }
    wave_sync();                                               // previous tile's LDS reads are done
    // ---- expand the 32 rows: sD[row, c] = sum_k (c_alpha U)[c, k] z[row, k], NTB column tiles at a time ----
    auto block = [&](int nt0, auto ntile_count) {
      constexpr int N = decltype(ntile_count)::value;
      v16f acc[N];
#pragma unroll
      for (int i = 0; i < N; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
      const float2* fb = fl + 16 * nt0;
#pragma unroll
      for (int j = 0; j < JT; ++j) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
          const float2 b2 = column_coef(fb[j * ld + 16 * i], part);
          acc[i] = mfma32(zcur[j].x, b2.x, acc[i]);
          acc[i] = mfma32(zcur[j].y, b2.y, acc[i]);
        }
      }
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const int c = 32 * (nt0 + i) + col;
        if (c < N2) {
#pragma unroll
          for (int r = 0; r < 16; ++r) sD[d_row(r, half) * N2 + c] = acc[i][r];
        }
      }
    };
    {
      int nt0 = 0;
      for (; nt0 + NTB <= NTm; nt0 += NTB) block(nt0, std::integral_constant<int, NTB>());
      if (NTB > 1)
        for (; nt0 < NTm; ++nt0) block(nt0, std::integral_constant<int, 1>());
    }
    if (vtail) {                                               // the last complex column, without the matrix cores
      const float2* ft = sF + half * JT * ld + (M - 1);
      float pre = 0.f, pim = 0.f;
#pragma unroll
      for (int jj = 0; jj < JT; ++jj) {
        const float2 cf = ft[jj * ld];
        pre += zcur[jj].x * cf.x - zcur[jj].y * cf.y;
        pim += zcur[jj].x * cf.y + zcur[jj].y * cf.x;
      }
      pre += __shfl_xor(pre, 32, 64);
      pim += __shfl_xor(pim, 32, 64);
      if (half == 0) *reinterpret_cast<float2*>(&sD[col * N2 + N2 - 2]) = make_float2(pre, pim);
    }
    wave_sync();
    // ---- AdamUpdate on the sparse values that live in this tile; add lambda N_S into the tile ----
    if (cj0 + lane < cj1) sparse_adam_entry(sp, cj0 + lane, c_om, c_g, c_m, c_v, w_base, sD);
    if (cj1 - cj0 > 64u)                                       // rare: more than 64 entries in one tile
      for (uint32_t j = cj0 + 64u + lane; j < cj1; j += 64)
        sparse_adam_entry(sp, j, sp.omega[j], sp.gs[j], sp.ms[j], sp.vs[j], w_base, sD);
    wave_sync();
    // ---- stream the tile into W ----
    claim_small();
#pragma unroll
    for (int i = 0; i < kPre; ++i) claim_raw(wpre[i]);
    const int nfull = n4 >> 6;                                 // pieces every lane owns: no per-lane branch
#pragma unroll
    for (int i = 0; i < kPre; ++i) {
      const int q = lane_now + i * 64;
      if (i < nfull || q < n4) nt_store(&w4[q], WS::apply(wpre[i], sD, q, decay));
    }
    for (int q = lane + kPre * 64; q < n4; q += 64) w4[q] = WS::apply(w4[q], sD, q, decay);
    {                                                          // elements past the last whole piece
      const int e = n4 * WS::kElems + lane;
      if (e < n_w) WS::apply_one(w, w_base + e, sD + 2 * e, decay);
    }
    if (nxt >= ntiles) break;
    tile = nxt;
    nxt = nn;
    cj0 = nj0;
    cj1 = nj1;
    nj0 = nnj0;
    nj1 = nnj1;
  }
}

// k_lupdate_fused: k_lupdate with the reconstruction stage of mode N-1 (extent 32 S, rank K2 <= 32)
// in front of it, so the tensor between the two stages never exists.  A wavefront walks whole
// slabs; per tile (32 rows i2 of the slab):
//   stage A   D'[(m3, p), i2] = sum_m2 Y1[m2, m3] U2[i2, m2]            (rows = interleaved (m3, p))
//             A operand: lane (rho = 2 m3 + p, half) holds Y1[2 jj + half][m3] (parts chosen per p and
//             per factor part: re(u y) = ur yr - ui yi, im(u y) = ur yi + ui yr),
//             B operand: U2[i2, 2 jj + half] from the packed copy `ut` (two steps per 16-byte load);
//   stage B   the accumulator registers of D' ARE the operand rows of the last-mode expansion: in lane
//             (i2, half) registers (2 u, 2 u + 1) hold (re, im) of element k = (u & 1) + 4 (u >> 1) + 2 half
//             of row i2, so step (u, part) pairs elements k(u, 0) and k(u, 1) and the coefficient
//             table is read at those rows.  Everything after that is k_lupdate.
struct FusedPrev {
  const float2* y1;     // input of the fused stage: element (slab, m2, m3) of the (slabs, K2, K) complex tensor lies at
                        // y1[slab * s_slab + m2 * s_m2 + (m3 / 2) * s_pair + (m3 & 1) * s_odd]
  const float2* ut;     // U^(N-1)[i2, m2], zero for m2 >= K2, in operand order (k_pack_fused_factor)
  int S;                // tiles per slab
  int K2;               // rank of mode N-1
  int64_t s_slab, s_m2, s_pair, s_odd;   // row-major: K2 K, K, 2, 1; one column pair at a time (k_core2<2>):
                                         // 2, (K / 2) slabs 2, slabs 2, 1; one column at a time (k_core2<1>):
                                         // 1, K slabs, 2 slabs, slabs
};

template <int WDT, int W, int MS, int JT2, int UP>
__global__ __launch_bounds__(64 * W, 2) void k_lupdate_fused(const float2* __restrict__ U, int64_t A, int K,
                                                             int M, int64_t ntiles, void* __restrict__ w,
                                                             float decay, float c_alpha, SparseAdam sp,
                                                             FusedPrev fz) {
  typedef WStore<WDT> WS;
  typedef typename WS::raw wraw;
  constexpr int kPre = WS::kElems == 2 ? UP : (UP + 1) / 2;   // 16-byte pieces of the W tile per lane in flight
  constexpr int T = 64 * W;
  extern __shared__ float smem[];
  // MS > 0: the extent of the last mode is the compile-time constant MS (the host passes M == MS): stage B
  // then runs without a single vector-ALU instruction between its matrix instructions (see below).
  const int N2 = MS > 0 ? 2 * MS : 2 * M;
  const int NT = (N2 + 31) >> 5;
  const int ld = 16 * NT;
  const int slice = (kTileRows * N2 + 3) & ~3;                 // floats per wavefront: flat image of its W tile
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  float* sD = smem + wave * slice;
  float2* sF = reinterpret_cast<float2*>(smem + W * slice);
  stage_factor_table<false>(sF, U, K, K, M, 16, ld, tid, T, c_alpha);   // 16 rows: K <= 16 here; scaled by c_alpha
  __syncthreads();                                             // the only workgroup barrier
  // A half-spectrum last mode has 2^m + 1 entries: its last complex column would occupy a whole
  // 32-column matrix-core tile on its own.  That column is expanded with ordinary arithmetic
  // instead: each lane holds 8 of the 16 elements of its row (see stage B), multiplies them with
  // the column's coefficients - which do not depend on the tile and stay in registers - and the
  // two halves of the wavefront are added with one lane exchange.
  const bool vtail = (N2 & 31) == 2;
  const int NTm = vtail ? NT - 1 : NT;                         // column tiles that go through the matrix cores
  float2 ctail[8];                                             // (MS > 0: read from the table when used; the registers
#pragma unroll                                                 //  hold the matrix-core coefficients instead)
  for (int u = 0; u < 8; ++u) {
    const int k = (u & 1) + 4 * (u >> 1) + 2 * (lane >> 5);
    ctail[u] = (MS == 0 && vtail) ? sF[k * ld + (M - 1)] : make_float2(0.f, 0.f);
  }

  // MS > 0: the stage-B coefficients of every column tile, already in the form the lane's column needs
  // (they do not depend on the tile), in registers for the whole kernel.
  constexpr int kNTmS = MS > 0 ? ((2 * MS) & 31) == 2 ? (2 * MS + 31) / 32 - 1 : (2 * MS + 31) / 32 : 1;
  float2 cregB[kNTmS][8];
  if constexpr (MS > 0) {
    const float2* fl0 = sF + (2 * (lane >> 5)) * ld + ((lane & 31) >> 1);
#pragma unroll
    for (int i = 0; i < kNTmS; ++i)
#pragma unroll
      for (int u = 0; u < 8; ++u)
        cregB[i][u] = column_coef(fl0[((u & 1) + 4 * (u >> 1)) * ld + 16 * i], lane & 1);
  }

  const int64_t Iw = A * M;
  const int tile_w = kTileRows * M;
  const int S = fz.S;
  const int I2 = 32 * S;
  const int64_t nslabs = ntiles / S;                           // A = slabs * 32 S exactly
  const int64_t nw = (int64_t)gridDim.x * W;
  int64_t slab = (int64_t)blockIdx.x * W + wave;
  if (W == 4 && fz.s_slab == 2 && (gridDim.x & 15) == 0) {
    // One column pair at a time, a 128-byte line of the operand tensor holds 8 consecutive slabs: the two
    // workgroups that share it are given block indices 8 apart, i.e. the same XCD under round-robin
    // dispatch, so that one L2 fetches the line for both (otherwise two do: 1.03 x the kernel's traffic).
    const int64_t b = blockIdx.x;
    slab = 8 * (8 * (b >> 4) + (b & 7)) + 4 * ((b >> 3) & 1) + wave;
  }
  int ts = 0;
  if (slab >= nslabs) return;
  auto advance = [&](int64_t& sl, int& t) {
    if (t + 1 < S) { t += 1; } else { t = 0; sl += nw; }
  };

  int32_t my_om = -1;
  float2 my_g = make_float2(0.f, 0.f), my_m = make_float2(0.f, 0.f);
  float my_v = 0.f;
  const int om_last = sp.k_last;
  // sparse state of a tile with support range [j0, j1): fetched one tile ahead; unconditional loads
  // (lanes without an entry read a clamped, valid position and ignore it)
  auto issue_sparse = [&](uint32_t j0, uint32_t j1) {
    const uint32_t j = j0 + lane;
    const uint32_t jc = j < j1 ? j : (uint32_t)om_last;
    my_om = j < j1 ? sp.omega[jc] : -1;
    my_g = sp.gs[jc];
    my_m = sp.ms[jc];
    my_v = sp.vs[jc];
  };
  auto claim_sparse = [&]() {
    asm volatile("" : "+v"(my_om), "+v"(my_g.x), "+v"(my_g.y), "+v"(my_m.x), "+v"(my_m.y), "+v"(my_v));
  };

  const int vzero = opaque_zero();
  // W goes through buffer descriptors (one per 4 pieces), range-checked by the hardware: no clamps
  // and no lane masks in the streaming phase.  Bytes of a tile from the first piece of each group on:
  constexpr int kWGroups = (kPre + 3) / 4;
  const uint32_t w_tile_bytes = (uint32_t)tile_w * (uint32_t)(16 / WS::kElems);
  uint32_t w_rest[kWGroups];
#pragma unroll
  for (int k = 0; k < kWGroups; ++k) {
    const uint32_t done = (uint32_t)(k * 4 * 64 * 16);
    w_rest[k] = __builtin_amdgcn_readfirstlane(w_tile_bytes > done ? w_tile_bytes - done : 0u);
  }
  const int voff_w = lane * 16;
  int64_t tile = slab * S;
  int64_t nslab = slab;
  int nts = ts;
  advance(nslab, nts);
  bool have_next = nslab < nslabs;
  int64_t nxt = have_next ? nslab * S + nts : tile;
  uint32_t cj0 = sp.tile_start[tile + vzero], cj1 = sp.tile_start[tile + 1 + vzero];
  uint32_t nj0 = sp.tile_start[nxt + vzero], nj1 = sp.tile_start[nxt + 1 + vzero];
  issue_sparse(cj0, cj1);
  claim_sparse();
  // Stage-A operand rows (the slab's Y1) stay in registers for all S tiles of a slab.  Those of the NEXT slab
  // are requested right after stage A of a slab's last tile, when the registers have just been used
  // for the last time: they then have a whole stage B and W phase to arrive, however the tensor is laid
  // out (one column pair at a time, a lane's 16 loads touch 16 cache lines each).  Unconditional
  // loads with clamped indices: clamped rows / columns meet zero coefficients.
  float2 y1[JT2];
  auto fetch_y1 = [&](int64_t sl, int ln) {
    const int c2 = ln & 31, h2 = ln >> 5;
    const int m3 = (c2 >> 1) < K ? (c2 >> 1) : K - 1;
    const float2* yp = fz.y1 + sl * fz.s_slab + (int64_t)(m3 >> 1) * fz.s_pair + (int64_t)(m3 & 1) * fz.s_odd;
#pragma unroll
    for (int jj = 0; jj < JT2; ++jj) {
      const int m2 = 2 * jj + h2;
      y1[jj] = yp[(int64_t)(m2 < fz.K2 ? m2 : fz.K2 - 1) * fz.s_m2];
    }
  };
  fetch_y1(slab, lane);
  while (true) {
    int lane_now = lane;                                       // opaque per-tile copy (see k_lproj)
    asm volatile("" : "+v"(lane_now));
    const int col = lane_now & 31, half = lane_now >> 5;
    const int part = col & 1;
    const int64_t w_base = tile * tile_w;
    const int n_w = (int)((Iw - w_base) < tile_w ? (Iw - w_base) : tile_w);
    wraw* w4 = WS::tile(w, w_base);
    const int n4 = n_w / WS::kElems;                           // tiles are whole here: 32 M elements, a multiple of 4
    const int32_t c_om = my_om;
    const float2 c_g = my_g, c_m = my_m;
    const float c_v = my_v;
    // ---- this tile's 32 columns of the factor copy (small, cache-resident), issued BEFORE the W pieces so
    //      that waiting for them leaves those in flight ----
    float2 u2[JT2];
    {
      const float4* up = reinterpret_cast<const float4*>(fz.ut) + (size_t)ts * 8 * 64 + lane_now;
#pragma unroll
      for (int jp = 0; jp < JT2 / 2; ++jp) {                   // two operand rows per 16-byte load
        const float4 f = up[jp * 64];
        u2[2 * jp] = make_float2(f.x, f.y);
        u2[2 * jp + 1] = make_float2(f.z, f.w);
      }
    }
    // ---- this tile's W pieces go in flight ----
    wraw wpre[kPre];
    const char* w_tile = reinterpret_cast<const char*>(w4);
#pragma unroll
    for (int k = 0; k < kWGroups; ++k) {                       // a descriptor per 4 pieces: immediates reach 4 KB
      const __amdgpu_buffer_rsrc_t r = raw_buffer(w_tile + k * 4 * 64 * 16, w_rest[k]);
#pragma unroll
      for (int i = 4 * k; i < 4 * k + 4 && i < kPre; ++i) buffer_piece_load(wpre[i], r, voff_w + (i - 4 * k) * 64 * 16);
    }
    // The stage-A operands are claimed here: the asm statements pin every load above them (memory
    // clobber) and every use below them, so the scheduler cannot interleave load - wait - MFMA.
#pragma unroll
    for (int jj = 0; jj < JT2; ++jj)
      asm volatile("" : "+v"(y1[jj].x), "+v"(y1[jj].y), "+v"(u2[jj].x), "+v"(u2[jj].y) : : "memory");
    // ---- stage A: D' = rows of the mode-(N-1) expansion for the 32 rows of the tile ----
    v16f dz;
#pragma unroll
    for (int r = 0; r < 16; ++r) dz[r] = 0.f;
    if (ts == 0) {
      // (wave-uniform) first tile of a slab: the rows just claimed become the two A operands of the lane's
      // row (rho = 2 m3 + p): re(u y) = ur yr - ui yi, im(u y) = ur yi + ui yr; once per slab, not per tile
#pragma unroll
      for (int jj = 0; jj < JT2; ++jj) {
        const float2 y = y1[jj];
        y1[jj].x = part ? y.y : y.x;
        y1[jj].y = part ? y.x : -y.y;
      }
    }
#pragma unroll
    for (int jj = 0; jj < JT2; ++jj) {
      dz = mfma32(y1[jj].x, u2[jj].x, dz);
      dz = mfma32(y1[jj].y, u2[jj].y, dz);
    }
    if (nts == 0 && have_next) fetch_y1(nslab, lane_now);      // (wave-uniform) the next tile opens a new slab
    // ---- the next tile's sparse state goes in flight ----
    int64_t nnslab = nslab;
    int nnts = nts;
    advance(nnslab, nnts);
    const bool have_nn = have_next && nnslab < nslabs;
    const int64_t nn = have_nn ? nnslab * S + nnts : nxt;
    issue_sparse(nj0, nj1);
    const uint32_t nnj0 = sp.tile_start[nn + vzero], nnj1 = sp.tile_start[nn + 1 + vzero];
    wave_sync();                                               // previous tile's LDS reads are done
    // ---- stage B: expand the last mode: sD[row, c] = sum_k (c_alpha U)[c, k] ..., NTB column tiles at a time ----
    const float2* fl = sF + (2 * half) * ld + (col >> 1);      // row k(u, half) = (u & 1) + 4 (u >> 1) + 2 half
    if constexpr (MS > 0) {
      // Straight-line: 16 matrix instructions per column tile with coefficients from registers, then the tile's
      // 16 result rows written at constant offsets from one lane address.  (A vector-ALU instruction between two fp32 matrix instructions waits for the matrix
      // pipe: selects, zeroing and register copies in this stage cost more than its matrix work.)
      constexpr int N2s = 2 * MS;
      float* sDl = sD + (4 * half) * N2s + col;
      auto chain = [&](int i) -> v16f {
        v16f zero;
#pragma unroll
        for (int r = 0; r < 16; ++r) zero[r] = 0.f;
        v16f acc = mfma32(dz[0], cregB[i][0].x, zero);
        acc = mfma32(dz[1], cregB[i][0].y, acc);
#pragma unroll
        for (int u = 1; u < 8; ++u) {
          acc = mfma32(dz[2 * u], cregB[i][u].x, acc);
          acc = mfma32(dz[2 * u + 1], cregB[i][u].y, acc);
        }
        return acc;
      };
      auto put = [&](const v16f& acc, int i) {
        if (32 * (i + 1) <= N2s || 32 * i + col < N2s) {
#pragma unroll
          for (int r = 0; r < 16; ++r) sDl[((r & 3) + 8 * (r >> 2)) * N2s + 32 * i] = acc[r];
        }
      };
#pragma unroll
      for (int i = 0; i < kNTmS; ++i) put(chain(i), i);
    } else {
      // one column tile at a time, its 8 coefficient pairs fetched while the previous tile is in the
      // matrix cores (the last tile re-reads itself)
      float2 cf[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) cf[u] = fl[((u & 1) + 4 * (u >> 1)) * ld];
      for (int nt0 = 0; nt0 < NTm; ++nt0) {
        float2 cn[8];
        const float2* fn = fl + 16 * (nt0 + 1 < NTm ? nt0 + 1 : nt0);
#pragma unroll
        for (int u = 0; u < 8; ++u) cn[u] = fn[((u & 1) + 4 * (u >> 1)) * ld];
        v16f acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float2 b2 = column_coef(cf[u], part);
          acc = mfma32(dz[2 * u], b2.x, acc);
          acc = mfma32(dz[2 * u + 1], b2.y, acc);
        }
        const int c = 32 * nt0 + col;
        if (c < N2) {
#pragma unroll
          for (int r = 0; r < 16; ++r) sD[d_row(r, half) * N2 + c] = acc[r];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) cf[u] = cn[u];
      }
    }
    if (vtail) {                                               // the last complex column, without the matrix cores
      float pre = 0.f, pim = 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float zr = dz[2 * u], zi = dz[2 * u + 1];
        const float2 ct = MS > 0 ? sF[((u & 1) + 4 * (u >> 1) + 2 * half) * ld + (MS - 1)] : ctail[u];
        pre += zr * ct.x - zi * ct.y;
        pim += zr * ct.y + zi * ct.x;
      }
      pre += __shfl_xor(pre, 32, 64);
      pim += __shfl_xor(pim, 32, 64);
      if (half == 0) *reinterpret_cast<float2*>(&sD[col * N2 + N2 - 2]) = make_float2(pre, pim);
    }
    wave_sync();
    // ---- AdamUpdate on the sparse values that live in this tile; add lambda N_S into the tile ----
    if (cj0 + lane < cj1) sparse_adam_entry(sp, cj0 + lane, c_om, c_g, c_m, c_v, w_base, sD);
    if (cj1 - cj0 > 64u)                                       // rare: more than 64 entries in one tile
      for (uint32_t j = cj0 + 64u + lane; j < cj1; j += 64)
        sparse_adam_entry(sp, j, sp.omega[j], sp.gs[j], sp.ms[j], sp.vs[j], w_base, sD);
    wave_sync();
    // ---- the wait point for everything still in flight, then stream the tile into W ----
    claim_sparse();
#pragma unroll
    for (int i = 0; i < kPre; ++i) claim_raw(wpre[i]);
#pragma unroll
    for (int k = 0; k < kWGroups; ++k) {                       // (pieces past the tile's end are dropped by the range check)
      const __amdgpu_buffer_rsrc_t r = raw_buffer(w_tile + k * 4 * 64 * 16, w_rest[k]);
#pragma unroll
      for (int i = 4 * k; i < 4 * k + 4 && i < kPre; ++i) {
        const int q = lane_now + i * 64;                       // (the LDS read stays inside the tile)
        buffer_piece_store(WS::apply(wpre[i], sD, q < n4 ? q : n4 - 1, decay), r, voff_w + (i - 4 * k) * 64 * 16);
      }
    }
    for (int q = lane + kPre * 64; q < n4; q += 64) w4[q] = WS::apply(w4[q], sD, q, decay);
    if (!have_next) break;
    tile = nxt;
    slab = nslab;
    ts = nts;
    nxt = nn;
    nslab = nnslab;
    nts = nnts;
    have_next = have_nn;
    cj0 = nj0;
    cj1 = nj1;
    nj0 = nnj0;
    nj1 = nnj1;
  }
}

// Kernel-ready copies of the mode-(N-1) factor for the fused stages:
//   fpad = conj(U[i2, m2]) (m2 < r, else 0; 32 columns), tile by tile in matrix-core operand order
//                                                               -> second compression stage in k_lproj
//   ut   = U[i2, m2] (m2 < r, else 0; 32 columns), tile by tile in matrix-core operand order
//                                                               -> first reconstruction stage in k_lupdate_fused
__global__ void k_pack_fused_factor(const float2* __restrict__ U, int I2, int r, float2* __restrict__ fpad,
                                    float2* __restrict__ ut) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= I2 * 32) return;
  const int i2 = e >> 5, m2 = e & 31;
  const float2 u = m2 < r ? U[(int64_t)i2 * r + m2] : make_float2(0.f, 0.f);
  // fpad in the order the second compression stage consumes it: tile ts = i2 / 32, row i2 % 32 =
  // d_row(rr, half), lane = 32 half + m2; slot [ts][rr / 2][lane][rr % 2], so that a lane fetches the
  // operands of two accumulator rows with one 16-byte load and a wavefront reads 1 KB contiguous
  const int ts = i2 >> 5, il = i2 & 31;
  const int half = (il >> 2) & 1, rr = (il & 3) + 4 * (il >> 3);
  fpad[(((size_t)ts * 8 + (rr >> 1)) * 64 + 32 * half + m2) * 2 + (rr & 1)] = make_float2(u.x, -u.y);
  // ut in the order the first reconstruction stage consumes it: step jj = m2 / 2 of the lane
  // (i2 % 32, m2 % 2); slot [ts][jj / 2][lane][jj % 2]
  const int jj = m2 >> 1;
  ut[(((size_t)ts * 8 + (jj >> 1)) * 64 + 32 * (m2 & 1) + il) * 2 + (jj & 1)] = u;
}

// tile_start[t] = #{ j : Omega_j < t * tile_elems }, t = 0 .. ntiles (Omega ascending).
__global__ void k_tile_offsets(const int32_t* __restrict__ omega, int64_t k, int64_t tile_elems,
                               int64_t ntiles, uint32_t* __restrict__ tile_start) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t > ntiles) return;
  const int64_t target = t * tile_elems;
  int64_t lo = 0, hi = k;                                      // first j in [0, k] with Omega_j >= target
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if ((int64_t)omega[mid] < target) lo = mid + 1; else hi = mid;
  }
  tile_start[t] = (uint32_t)lo;
}

inline uint32_t magic_for(int d) {
  return d <= 1 ? 0u : (uint32_t)((0x100000000ull + (uint64_t)d - 1) / (uint64_t)d);
}

constexpr size_t kLdsLimit = 160 * 1024;

template <typename Kern>
bool allow_lds(Kern kern, size_t bytes) {
  if (bytes <= 48 * 1024) return true;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)bytes) == hipSuccess;
}

// Workgroups of `kern` that are resident on one compute unit at a time (registers, LDS), asked of
// the runtime once per kernel and LDS size.  The tile loops are persistent (stride = grid size), so
// the grid is exactly one resident set: more workgroups would run as a ragged second round.
template <typename Kern>
int resident_blocks(Kern kern, int threads, size_t lds) {
  static std::mutex mu;
  static std::map<std::pair<const void*, size_t>, int> cache;
  const std::pair<const void*, size_t> key(reinterpret_cast<const void*>(kern), lds);
  std::lock_guard<std::mutex> lock(mu);
  auto it = cache.find(key);
  if (it != cache.end()) return it->second;
  int nb = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, threads, lds) != hipSuccess || nb < 1) nb = 1;
  if (nb > 4) nb = 4;
  cache[key] = nb;
  return nb;
}

// Compute units of the current device (256 on an MI355X), asked of the runtime once per device.
int compute_units() {
  constexpr int kMaxDev = 64;
  static std::atomic<int> cached[kMaxDev];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) dev = 0;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
  cached[dev].store(n, std::memory_order_relaxed);
  return n;
}

int grid_for_tiles(int64_t ntiles, int blocks_per_cu) {
  const int64_t cap = (int64_t)compute_units() * blocks_per_cu;
  return (int)(ntiles < cap ? ntiles : cap);
}

}  // namespace

// ---- host side ---------------------------------------------------------------------------------

size_t lproj_lds_bytes(int W, int K, int M) {
  const int stride = 2 * K + ((K & 1) ? 0 : 2), J = (K + 1) / 2, NT = (2 * M + 31) / 32;
  return (size_t)W * (kTileRows * stride + 2) * 4 + (size_t)2 * J * 16 * NT * 8;
}

int lupdate_jt(int K) {                         // operand-register pairs per lane: power of two >= K / 2
  int jt = 1;
  while (2 * jt < K) jt *= 2;
  return jt;
}

size_t lupdate_lds_bytes(int W, int K, int M) {
  const int NT = (2 * M + 31) / 32;
  return (size_t)W * ((kTileRows * 2 * M + 3) & ~3) * 4 + (size_t)2 * lupdate_jt(K) * 16 * NT * 8;
}

constexpr int kUpdMaxJT = 16;                   // k_lupdate keeps a row of z in registers: rank of the last mode <= 32

// Wavefronts per workgroup for the two last-mode kernels (each wavefront stages its own 32-row
// tile in LDS), or 0 if the shape is outside what they cover.  `Klast` / `rlast` are the extent
// and the rank of the last mode.  Two workgroups per compute unit are preferred.
int fused_max_last_extent() { return 2 * kCoefPairs; }

int choose_tile_waves(int Klast, int rlast, int prefer) {
  if (lupdate_jt(rlast) > kUpdMaxJT) return 0;
  if (Klast < 2) return 0;                      // the tile loaders assume at least one 2-element piece per tile
  if ((int64_t)kTileRows * Klast >= (1 << 17)) return 0;
  const int cand[3] = {4, 2, 1};
  for (int pass = 0; pass < 2; ++pass) {
    const size_t limit = pass == 0 ? kLdsLimit / 2 : kLdsLimit;
    for (int i = 0; i < 3; ++i) {
      const int W = cand[i];
      if (W > prefer) continue;
      if (lproj_lds_bytes(W, Klast, rlast) <= limit && lupdate_lds_bytes(W, rlast, Klast) <= limit) return W;
    }
  }
  return 0;
}

// Launches one of the matrix-core loops over the whole chip (two workgroups of four wavefronts per compute
// unit); returns the real floating-point operations of the launch.
double launch_mfma_probe(hipStream_t s, int kind, int64_t iters, float* sink) {
  const int grid = compute_units() * 2;
  iters = (iters + kProbeUnroll - 1) / kProbeUnroll * kProbeUnroll;
  const double instr = (double)grid * 4.0 * (double)iters * kProbeChains;
  if (kind == 0) {
    k_mfma_probe_f32<<<dim3((unsigned)grid), dim3(256), 0, s>>>(sink, iters, 1.f, 0.5f);
    return instr * 4096.0;                                     // 32 x 32 x 2 multiply-adds
  }
  k_mfma_probe_f64<<<dim3((unsigned)grid), dim3(256), 0, s>>>(sink, iters, 1., 0.5);
  return instr * 2048.0;                                       // 16 x 16 x 4 multiply-adds
}

void launch_tile_offsets(hipStream_t s, const int32_t* omega, int64_t k, int64_t tile_elems,
                         int64_t ntiles, uint32_t* tile_start) {
  const int64_t n = ntiles + 1;
  k_tile_offsets<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(omega, k, tile_elems, ntiles,
                                                                        tile_start);
}

void launch_mid(hipStream_t s, const float2* x, const float2* U, int rn, bool project, const Stage& st,
                float2* out) {
  const int64_t A = st.A, B = st.B;
  const int K = st.K, M = st.M;
  if (A * M * B <= 0) return;
  const int vec = (B % 2 == 0) ? 2 : 1;
  const int64_t ncv = A * (B / vec);
  const int J = (K + 1) / 2;
  const int jn = J < kMidJChunk ? J : kMidJChunk;
  // Fewer workgroups than compute units: share 32 columns between the 4 wavefronts of a workgroup
  // (MODE 1 / 2) so that the stage still spreads over the chip; otherwise every wavefront owns 32
  // columns (MODE 0; measured faster as soon as it yields at least one workgroup per compute unit).
  const int mt0 = M > 32 ? 2 : 1;
  const int64_t wgs0 = ((ncv + 127) / 128) * ((M + 32 * mt0 - 1) / (32 * mt0));
  int mode = 0;
  if (wgs0 < compute_units()) mode = M > 32 ? 2 : 1;
  const int mt = mode == 0 ? mt0 : 1;
  const int tl = mode == 2 ? 4 : mt;
  const int64_t gx = mode == 0 ? (ncv + 127) / 128 : (ncv + 31) / 32;
  const int gy = (M + 32 * tl - 1) / (32 * tl);
  size_t lds = (size_t)jn * tl * 64 * 8;
  if (mode == 1) {
    const size_t red = (size_t)3 * 2 * vec * 16 * 64 * 4;
    if (red > lds) lds = red;
  }
  dim3 grid((unsigned)gx, (unsigned)gy), block(kMidThreads);
  const float* xf = reinterpret_cast<const float*>(x);
  float* of = reinterpret_cast<float*>(out);
#define TGRAD_MID(MT_, VEC_, P_, MODE_)                                                   \
  do {                                                                                    \
    allow_lds(k_mid<MT_, VEC_, P_, MODE_>, lds);                                          \
    k_mid<MT_, VEC_, P_, MODE_><<<grid, block, lds, s>>>(xf, U, rn, A, K, M, B, of);      \
  } while (0)
#define TGRAD_MID_P(MT_, VEC_, MODE_)                                                     \
  do {                                                                                    \
    if (project) TGRAD_MID(MT_, VEC_, true, MODE_); else TGRAD_MID(MT_, VEC_, false, MODE_); \
  } while (0)
  if (mode == 0) {
    if (mt == 1) { if (vec == 2) TGRAD_MID_P(1, 2, 0); else TGRAD_MID_P(1, 1, 0); }
    else         { if (vec == 2) TGRAD_MID_P(2, 2, 0); else TGRAD_MID_P(2, 1, 0); }
  } else if (mode == 1) {
    if (vec == 2) TGRAD_MID_P(1, 2, 1); else TGRAD_MID_P(1, 1, 1);
  } else {
    if (vec == 2) TGRAD_MID_P(1, 2, 2); else TGRAD_MID_P(1, 1, 2);
  }
#undef TGRAD_MID_P
#undef TGRAD_MID
}

// Limits of k_core: one 32-row tile of core rows, and LDS for both operand tables.
bool core_kernel_fits(int K, int M) { return M >= 1 && M <= 32 && K >= 1 && K <= TGRAD_MAX_EXTENT; }

// Last compression stage + AdamUpdate on the core + first reconstruction stage (mode 1: the tensor
// before is (K, B), the tensor after is (K, B) again, the core in between (M, B)).
void launch_core(hipStream_t s, const float2* x, const float2* U, int rn, int K, int M, int64_t B, float2* m,
                 float* v, float2* g_out, float beta1, float beta2, float inv_c1, float inv_c2, float eps,
                 float2* z) {
  if (B <= 0) return;
  const int vec = (B % 2 == 0) ? 2 : 1;
  const int64_t BV = B / vec;
  const int J = (K + 1) / 2, NTI = (K + 31) / 32;
  const size_t red = (size_t)4 * 2 * vec * 16 * 64 / 2;
  const size_t lds = (((size_t)J * 64 > red ? (size_t)J * 64 : red) + (size_t)16 * NTI * 64) * 8;
  dim3 grid((unsigned)((BV + 31) / 32)), block(kMidThreads);
  CoreAdam ad{m, v, g_out, beta1, beta2, inv_c1, inv_c2, eps};
  const float* xf = reinterpret_cast<const float*>(x);
  float* zf = reinterpret_cast<float*>(z);
  if (vec == 2) {
    allow_lds(k_core<2>, lds);
    k_core<2><<<grid, block, lds, s>>>(xf, U, rn, K, M, B, ad, zf);
  } else {
    allow_lds(k_core<1>, lds);
    k_core<1><<<grid, block, lds, s>>>(xf, U, rn, K, M, B, ad, zf);
  }
}

// Limits of k_core2: first extent 128 (one 32-row tile per wavefront), ranks within one tile, the second
// extent within four tiles, and enough column groups (one workgroup each) to occupy the chip: pairs of
// columns if there are at least 192 pairs (3/4 of the 256 compute units of the MI355X; the rank of the
// last mode must then be even: a pair lies inside one row of the mode before it), else single columns if
// there are at least 96.  Below that the three separate kernels, which spread over the chip, are
// faster.  Returns the columns per workgroup (2 or 1), or 0.  A function of the shape alone: the
// workspace layout follows from it, and the size query must not depend on the device that is current.
constexpr int64_t kCore2MinPairs = 192, kCore2MinColumns = 96;
int core2_kernel_vec(int I0, int I1, int M0, int M1, int K2, int K) {
  const int64_t Cc = (int64_t)K2 * K;
  if (!(I0 == kCore2Rows && I1 >= 1 && I1 <= 128 && M0 >= 1 && M0 <= 32 && M1 >= 1 && M1 <= 32 &&
        (int64_t)I0 * I1 * Cc < ((int64_t)1 << 28)))
    return 0;
  if (K % 2 == 0 && Cc / 2 >= kCore2MinPairs) return 2;
  if (Cc >= kCore2MinColumns) return 1;
  return 0;
}

size_t core2_table_bytes(int I1) { return (size_t)core2_table_elems(I1) * 8; }

// The factors of the two leading modes in the operand order of k_core2's four stages (once per refresh).
void launch_pack_core2(hipStream_t s, const float2* U0, int rn0, int M0, const float2* U1, int rn1, int M1, int I1,
                       float2* tab) {
  const int n = core2_table_elems(I1);
  k_pack_core2<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(U0, rn0, M0, U1, rn1, M1, I1, tab);
}

// The two leading modes compressed, AdamUpdate on the core, the two leading modes reconstructed:
// x (128, I1, Cc) -> z (Cc / zgroup, 128, I1) units of zgroup complex (zgroup = vec, or 2 with vec = 1 and Cc
// even), the core (M0, M1, Cc) in between.
void launch_core2(hipStream_t s, int vec, int zgroup, const float2* x, const float2* tab, int I1, int M0, int M1, int64_t Cc,
                  float2* m, float* v, float2* g_out, float beta1, float beta2, float inv_c1, float inv_c2,
                  float eps, float2* z) {
  const int NT1 = (I1 + 31) / 32;
  const size_t lds = (size_t)64 * 1024 + (size_t)NT1 * 16 * 64 * 8;
  Core2Args a{reinterpret_cast<const float*>(x), reinterpret_cast<float*>(z), tab, I1, M0, M1, Cc, zgroup};
  CoreAdam ad{m, v, g_out, beta1, beta2, inv_c1, inv_c2, eps};
  if (vec == 2) {
    allow_lds(k_core2<2>, lds);
    k_core2<2><<<dim3((unsigned)(Cc / 2)), dim3(kMidThreads), lds, s>>>(a, ad);
  } else {
    allow_lds(k_core2<1>, lds);
    k_core2<1><<<dim3((unsigned)Cc), dim3(kMidThreads), lds, s>>>(a, ad);
  }
}

void launch_pack_fused_factor(hipStream_t s, const float2* U, int I2, int r, float2* fpad, float2* ut) {
  k_pack_fused_factor<<<dim3((unsigned)((I2 * 32 + 255) / 256)), dim3(256), 0, s>>>(U, I2, r, fpad, ut);
}

// `fused_I2` > 0: also contract the next mode (extent fused_I2 = 32 S, rank fused_M2, factor copy
// `fpad`) and write its result to `out` (slabs, fused_M2, M); otherwise `out` is (A, M).
void launch_lproj(hipStream_t s, const void* g, int dtype, const int32_t* omega, const uint32_t* tile_start,
                  float2* gs, const float2* U, int rn, const Stage& st, int W, float2* out, int fused_I2,
                  int fused_M2, const float2* fpad) {
  const int64_t A = st.A;
  const int K = st.K, M = st.M;
  if (A * M <= 0) return;
  const int64_t ntiles = (A + kTileRows - 1) / kTileRows;
  const size_t lds = lproj_lds_bytes(W, K, M);
  const int NT = (2 * M + 31) / 32;
  const int ntb = NT >= 2 ? 2 : 1;
  const bool fuse = fused_I2 > 0;
  const int S = fuse ? fused_I2 / kTileRows : 1;
  const int64_t nslabs = (ntiles + S - 1) / S;
  const int tb = (K + 3) / 4 <= 5 ? 5 : (K + 3) / 4 <= 9 ? 9 : kTileBatch;   // pieces per lane a tile needs (capped)
  const int64_t ngroups = (nslabs + W - 1) / W;                // workgroups' worth of tile sequences
  dim3 grid(1), block(64 * W);
  float* of = reinterpret_cast<float*>(out);
  const uint32_t magic = magic_for(K);
  FusedNext fz{fpad, of, S, fused_M2};
#define TGRAD_LP_C(DT_, W_, NTB_, F_, Z_, CP_, TB_)                                                      \
  do {                                                                                                   \
    allow_lds(k_lproj<DT_, W_, NTB_, F_, Z_, CP_, TB_>, lds);                                            \
    grid.x = (unsigned)grid_for_tiles(ngroups, resident_blocks(k_lproj<DT_, W_, NTB_, F_, Z_, CP_, TB_>, 64 * W_, lds)); \
    k_lproj<DT_, W_, NTB_, F_, Z_, CP_, TB_><<<grid, block, lds, s>>>(g, omega, tile_start, gs, U, rn,   \
                                                                      A, K, M, magic, ntiles, of, fz);   \
  } while (0)
#define TGRAD_LP(DT_, W_, NTB_, F_) TGRAD_LP_C(DT_, W_, NTB_, F_, false, 1, kTileBatch)
#define TGRAD_LP_FUSED(DT_, F_)                                                                          \
  do {                                                                                                   \
    if ((K + 1) / 2 > kCoefPairsShort) TGRAD_LP_C(DT_, 4, 1, F_, true, kCoefPairs, kTileBatch);          \
    else if (tb == 5) TGRAD_LP_C(DT_, 4, 1, F_, true, kCoefPairsShort, 5);                               \
    else TGRAD_LP_C(DT_, 4, 1, F_, true, kCoefPairsShort, 9);                                            \
  } while (0)
#define TGRAD_LP_F(DT_, W_, NTB_)                                                                        \
  do {                                                                                                   \
    if (K & 1) TGRAD_LP(DT_, W_, NTB_, true); else TGRAD_LP(DT_, W_, NTB_, false);                       \
  } while (0)
#define TGRAD_LP_F4(DT_, NTB_)   /* 4 wavefronts: also the variants for narrow last modes */              \
  do {                                                                                                   \
    if (tb == kTileBatch) TGRAD_LP_F(DT_, 4, NTB_);                                                      \
    else if (tb == 9) { if (K & 1) TGRAD_LP_C(DT_, 4, NTB_, true, false, 1, 9); else TGRAD_LP_C(DT_, 4, NTB_, false, false, 1, 9); } \
    else { if (K & 1) TGRAD_LP_C(DT_, 4, NTB_, true, false, 1, 5); else TGRAD_LP_C(DT_, 4, NTB_, false, false, 1, 5); } \
  } while (0)
#define TGRAD_LP_W(DT_, NTB_)                                                                            \
  do {                                                                                                   \
    if (W == 4) TGRAD_LP_F4(DT_, NTB_); else if (W == 2) TGRAD_LP_F(DT_, 2, NTB_); else TGRAD_LP_F(DT_, 1, NTB_); \
  } while (0)
#define TGRAD_LPF_C(DT_, CP_, TB_)                                                                       \
  do {                                                                                                   \
    const size_t ldsf = (size_t)4 * lproj_flat_slice(K, TB_) * 4 + (size_t)2 * ((K + 1) / 2) * 16 * 8;   \
    allow_lds(k_lproj_flat<DT_, CP_, TB_>, ldsf);                                                        \
    grid.x = (unsigned)grid_for_tiles(ngroups, resident_blocks(k_lproj_flat<DT_, CP_, TB_>, 256, ldsf)); \
    k_lproj_flat<DT_, CP_, TB_><<<grid, block, ldsf, s>>>(g, omega, tile_start, gs, U, rn, A, K, M,      \
                                                          ntiles, fz);                                   \
  } while (0)
#define TGRAD_LPF(DT_)                                                                                   \
  do {                                                                                                   \
    if ((K + 1) / 2 > kCoefPairsShort) TGRAD_LPF_C(DT_, kCoefPairs, kTileBatch);                         \
    else if (tb == 5) TGRAD_LPF_C(DT_, kCoefPairsShort, 5);                                              \
    else TGRAD_LPF_C(DT_, kCoefPairsShort, 9);                                                           \
  } while (0)
  const int cp = (K + 1) / 2 > kCoefPairsShort ? kCoefPairs : kCoefPairsShort;
  if (fuse && (K & 1) && tb * 64 >= 16 * K && 62 * K + 4 * cp <= tb * 256) {   // odd last extent: the staging phase without vector ALU work
    if (dtype == TGRAD_C64) TGRAD_LPF(TGRAD_C64); else TGRAD_LPF(TGRAD_CBF16);
  } else if (fuse) {                            // the host only fuses with W == 4 and one column tile
    if (dtype == TGRAD_C64) {
      if (K & 1) TGRAD_LP_FUSED(TGRAD_C64, true); else TGRAD_LP_FUSED(TGRAD_C64, false);
    } else {
      if (K & 1) TGRAD_LP_FUSED(TGRAD_CBF16, true); else TGRAD_LP_FUSED(TGRAD_CBF16, false);
    }
  } else if (dtype == TGRAD_C64) {
    if (ntb == 2) TGRAD_LP_W(TGRAD_C64, 2); else TGRAD_LP_W(TGRAD_C64, 1);
  } else {
    if (ntb == 2) TGRAD_LP_W(TGRAD_CBF16, 2); else TGRAD_LP_W(TGRAD_CBF16, 1);
  }
#undef TGRAD_LPF
#undef TGRAD_LPF_C
#undef TGRAD_LP_F4
#undef TGRAD_LP_W
#undef TGRAD_LP_F
#undef TGRAD_LP_FUSED
#undef TGRAD_LP
#undef TGRAD_LP_C
}

void launch_lupdate(hipStream_t s, const float2* z, const float2* U, const Stage& st, int W, void* w,
                    int wdtype, float decay, float c_alpha, const int32_t* omega, const uint32_t* tile_start,
                    const float2* gs, float2* ms, float* vs, float beta1, float beta2, float inv_c1,
                    float inv_c2, float eps, float c_lambda) {
  const int64_t A = st.A;
  const int K = st.K, M = st.M;
  if (A * M <= 0) return;
  const int64_t ntiles = (A + kTileRows - 1) / kTileRows;
  const size_t lds = lupdate_lds_bytes(W, K, M);
  const int64_t ngroups = (ntiles + W - 1) / W;
  dim3 grid(1), block(64 * W);
  SparseAdam sp{omega, tile_start, gs, ms, vs, beta1, beta2, inv_c1, inv_c2, eps, c_lambda, 0};
  const float* zf = reinterpret_cast<const float*>(z);
  const int jt = lupdate_jt(K);
  const int up = (M + 3) / 4 <= 5 ? 5 : (M + 3) / 4 <= 9 ? 9 : kUpdPrefetch;
#define TGRAD_LU_U(W_, JT_, UP_)                                                                         \
  do {                                                                                                   \
    if (wdtype == TGRAD_C64) {                                                                           \
      allow_lds(k_lupdate<TGRAD_C64, W_, 2, JT_, UP_>, lds);   \
      grid.x = (unsigned)grid_for_tiles(ngroups, resident_blocks(k_lupdate<TGRAD_C64, W_, 2, JT_, UP_>, 64 * W_, lds));                                             \
      k_lupdate<TGRAD_C64, W_, 2, JT_, UP_><<<grid, block, lds, s>>>(zf, U, A, K, M, ntiles, w, decay, c_alpha, sp); \
    } else {                                                                                             \
      allow_lds(k_lupdate<TGRAD_CBF16, W_, 2, JT_, UP_>, lds);   \
      grid.x = (unsigned)grid_for_tiles(ngroups, resident_blocks(k_lupdate<TGRAD_CBF16, W_, 2, JT_, UP_>, 64 * W_, lds));                                           \
      k_lupdate<TGRAD_CBF16, W_, 2, JT_, UP_><<<grid, block, lds, s>>>(zf, U, A, K, M, ntiles, w, decay, c_alpha, sp); \
    }                                                                                                    \
  } while (0)
#define TGRAD_LU(W_, JT_)        /* 4 wavefronts: also the variants for narrow last modes */              \
  do {                                                                                                   \
    if (W_ == 4 && up == 5) TGRAD_LU_U(4, JT_, 5);                                                       \
    else if (W_ == 4 && up == 9) TGRAD_LU_U(4, JT_, 9);                                                  \
    else TGRAD_LU_U(W_, JT_, kUpdPrefetch);                                                              \
  } while (0)
#define TGRAD_LU_J(W_)                                                                                   \
  do {                                                                                                   \
    if (jt <= 1) TGRAD_LU(W_, 1); else if (jt == 2) TGRAD_LU(W_, 2); else if (jt == 4) TGRAD_LU(W_, 4);  \
    else if (jt == 8) TGRAD_LU(W_, 8); else TGRAD_LU(W_, 16);                                            \
  } while (0)
  if (W == 4) TGRAD_LU_J(4); else if (W == 2) TGRAD_LU_J(2); else TGRAD_LU_J(1);
#undef TGRAD_LU_U
#undef TGRAD_LU_J
#undef TGRAD_LU
}

// k_lupdate with the reconstruction stage of mode N-1 in front (see k_lupdate_fused): `y1` is the
// tensor before that stage, (slabs, K2, K) complex (`group` = 0) - or the same tensor one column group at
// a time: (K2 K / group, slabs) units of `group` = 1 or 2 neighbouring complex numbers (2: K even);
// `ut` the transposed factor copy; I2 = 32 S.
void launch_lupdate_fused(hipStream_t s, const float2* y1, const float2* ut, int I2, int K2, const float2* U,
                          const Stage& st, void* w, int wdtype, float decay, float c_alpha, const int32_t* omega,
                          const uint32_t* tile_start, int64_t k, const float2* gs, float2* ms, float* vs,
                          float beta1, float beta2, float inv_c1, float inv_c2, float eps, float c_lambda,
                          int group) {
  const int64_t A = st.A;
  const int K = st.K, M = st.M;
  if (A * M <= 0) return;
  constexpr int W = 4;
  const int64_t ntiles = A / kTileRows;
  const int S = I2 / kTileRows;
  const int64_t nslabs = ntiles / S;
  const int NT = (2 * M + 31) / 32;
  const size_t lds = (size_t)W * ((kTileRows * 2 * M + 3) & ~3) * 4 + (size_t)16 * 16 * NT * 8;
  const int64_t ngroups = (nslabs + W - 1) / W;
  dim3 grid(1), block(64 * W);
  SparseAdam sp{omega, tile_start, gs, ms, vs, beta1, beta2, inv_c1, inv_c2, eps, c_lambda,
                (int)(k > 0 ? k - 1 : 0)};
  FusedPrev fz{y1, ut, S, K2, (int64_t)K2 * K, (int64_t)K, 2, 1};
  if (group == 2) {                              // (K2 K / 2, slabs) units of two complex: what k_core2<2> writes
    fz.s_slab = 2;
    fz.s_pair = nslabs * 2;
    fz.s_m2 = (int64_t)(K / 2) * nslabs * 2;
  } else if (group == 1) {                       // (K2 K, slabs) complex: what k_core2<1> writes
    fz.s_slab = 1;
    fz.s_odd = nslabs;
    fz.s_pair = nslabs * 2;
    fz.s_m2 = (int64_t)K * nslabs;
  }
  const int up = (M + 3) / 4 <= 5 ? 5 : (M + 3) / 4 <= 9 ? 9 : kUpdPrefetch;
#define TGRAD_LUF_M(JT2_, UP_, MS_)                                                                      \
  do {                                                                                                   \
    if (wdtype == TGRAD_C64) {                                                                           \
      allow_lds(k_lupdate_fused<TGRAD_C64, W, MS_, JT2_, UP_>, lds);                                     \
      grid.x = (unsigned)grid_for_tiles(ngroups, resident_blocks(k_lupdate_fused<TGRAD_C64, W, MS_, JT2_, UP_>, 64 * W, lds)); \
      k_lupdate_fused<TGRAD_C64, W, MS_, JT2_, UP_><<<grid, block, lds, s>>>(U, A, K, M, ntiles, w, decay, c_alpha, sp, fz); \
    } else {                                                                                             \
      allow_lds(k_lupdate_fused<TGRAD_CBF16, W, MS_, JT2_, UP_>, lds);                                   \
      grid.x = (unsigned)grid_for_tiles(ngroups, resident_blocks(k_lupdate_fused<TGRAD_CBF16, W, MS_, JT2_, UP_>, 64 * W, lds)); \
      k_lupdate_fused<TGRAD_CBF16, W, MS_, JT2_, UP_><<<grid, block, lds, s>>>(U, A, K, M, ntiles, w, decay, c_alpha, sp, fz); \
    }                                                                                                    \
  } while (0)
  // the half-spectrum extents of FNO layers (2^m + 1) get a stage B with the extent as a compile-time constant
#define TGRAD_LUF_U(JT2_, UP_, MS_)                                                                      \
  do {                                                                                                   \
    if (M == MS_) TGRAD_LUF_M(JT2_, UP_, MS_); else TGRAD_LUF_M(JT2_, UP_, 0);                           \
  } while (0)
#define TGRAD_LUF(JT2_)                                                                                  \
  do {                                                                                                   \
    if (up == 5) TGRAD_LUF_U(JT2_, 5, 17); else if (up == 9) TGRAD_LUF_U(JT2_, 9, 33);                   \
    else TGRAD_LUF_U(JT2_, kUpdPrefetch, 65);                                                            \
  } while (0)
  if (K2 <= 8) TGRAD_LUF(4); else if (K2 <= 16) TGRAD_LUF(8); else TGRAD_LUF(16);
#undef TGRAD_LUF_U
#undef TGRAD_LUF_M
#undef TGRAD_LUF
}

}  // namespace tgrad
