// Factor refresh: {U^(n)} <- TuckerFactors(R_L, r), third line of the refresh branch of
// Algorithm 1, as HOSVD (appendix "Implementation": truncated SVD of every mode-n unfolding).
// The left singular vectors of the unfolding R_L(n) are the eigenvectors of the Hermitian
// mode-n Gram matrix A_n = R_L(n) R_L(n)^H, so the refresh is
//   (1) A_n for every compressed mode, accumulated in float64 on the f64 matrix cores, with
//       R_L = G - Sparse(G, Omega) formed on load from the support bitmask, and
//   (2) a cyclic Jacobi eigen-solve of each A_n in float64 (one workgroup per mode), the
//       r_n leading eigenvectors written eigenvalue-descending with the phase of every column
//       fixed (largest-modulus entry real and positive).
// float64 is used because Adam in core space is not invariant to the basis inside the subspace:
// noise-like gradients have relative eigenvalue gaps near 1e-4, and float32 accumulation error
// divided by such a gap would move the individual eigenvectors far more than the update tolerates.
#include "device_common.h"

namespace tgrad {

namespace {

typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int kSuper = 128;          // rows of the output handled by one workgroup, per side
constexpr int kTC = 16;              // tensor columns staged per tile
constexpr int kLd = kTC + 1;         // padded LDS row stride (float2 units), odd -> conflict-free
constexpr int kGramThreads = 1024;   // 16 wavefronts: a 4 x 4 grid of 32 x 32 output blocks

// Gram of the tensor viewed as (A, In, B): gram[i, j] = sum_{a, b} x[a, i, b] conj(x[a, j, b]).
// Real embedding on v_mfma_f64_16x16x4f64 (K = 4 = two tensor columns x {re, im}):
//   Re[i, j] = sum xr_i xr_j + xi_i xi_j      -> A operand (xr_i | xi_i),  B operand (xr_j | xi_j)
//   Im[i, j] = sum xi_i xr_j - xr_i xi_j      -> A operand (xi_i | -xr_i), B operand (xr_j | xi_j)
// Operand lanes: A[i = lane % 16][k = lane / 16], B[k = lane / 16][j = lane % 16];
// result: register r of lane l holds D[4 r + l / 16][l % 16].
// Workgroup (chunk, super-tile pair) writes its 128 x 128 block of partials[chunk].
template <int DT>
__global__ __launch_bounds__(kGramThreads) void k_gram(const void* __restrict__ x,
                                                        const uint32_t* __restrict__ mask, int64_t A,
                                                        int In, int64_t B, int64_t cols_per_chunk,
                                                        double* __restrict__ partials) {
  __shared__ float2 sI[kSuper * kLd];
  __shared__ float2 sJ[kSuper * kLd];
  const int nsup = (In + kSuper - 1) / kSuper;
  const int si = blockIdx.y / nsup, sj = blockIdx.y % nsup;
  const float2* sJp = (si == sj) ? sI : sJ;
  const int64_t J = A * B;
  const int64_t c_begin = (int64_t)blockIdx.x * cols_per_chunk;
  const int64_t c_end = c_begin + cols_per_chunk < J ? c_begin + cols_per_chunk : J;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int ri0 = (wave >> 2) * 32, rj0 = (wave & 3) * 32;
  const bool active = (si * kSuper + ri0 < In) && (sj * kSuper + rj0 < In);
  const int part = (lane >> 4) & 1;
  const int ccol = lane >> 5;
  const int lrow = lane & 15;

  v4d accRe[2][2], accIm[2][2];
  for (int a = 0; a < 2; ++a)
    for (int b = 0; b < 2; ++b) {
      accRe[a][b] = (v4d){0., 0., 0., 0.};
      accIm[a][b] = (v4d){0., 0., 0., 0.};
    }

  for (int64_t c0 = c_begin; c0 < c_end; c0 += kTC) {
    __syncthreads();                                  // previous tile fully consumed
    // ---- stage rows [s*128, s*128+128) x columns [c0, c0+16) for both sides ----
    for (int side = 0; side < ((si == sj) ? 1 : 2); ++side) {
      float2* dst = side == 0 ? sI : sJ;
      const int s = side == 0 ? si : sj;
      for (int e = tid; e < kSuper * kTC; e += kGramThreads) {
        int il, cl;
        if (B == 1) {                                 // rows are the fastest index in memory
          il = e % kSuper;
          cl = e / kSuper;
        } else {                                      // columns b are the fastest index
          il = e / kTC;
          cl = e % kTC;
        }
        const int i = s * kSuper + il;
        const int64_t c = c0 + cl;
        float2 v = make_float2(0.f, 0.f);
        if (i < In && c < c_end) {
          const int64_t a = c / B, b = c - a * B;
          const int64_t idx = (a * In + i) * B + b;
          bool drop = false;
          if (mask) drop = (mask[idx >> 5] >> (idx & 31)) & 1u;
          if (!drop) v = load_elem<DT>(x, idx);
        }
        dst[il * kLd + cl] = v;
      }
    }
    __syncthreads();
    if (active) {
#pragma unroll
      for (int s2 = 0; s2 < kTC / 2; ++s2) {
        const int cc = 2 * s2 + ccol;
        double aRe[2], aIm[2], bop[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          float2 xa = sI[(ri0 + t * 16 + lrow) * kLd + cc];
          float2 xb = sJp[(rj0 + t * 16 + lrow) * kLd + cc];
          aRe[t] = part ? (double)xa.y : (double)xa.x;
          aIm[t] = part ? -(double)xa.x : (double)xa.y;
          bop[t] = part ? (double)xb.y : (double)xb.x;
        }
#pragma unroll
        for (int ti = 0; ti < 2; ++ti)
#pragma unroll
          for (int tj = 0; tj < 2; ++tj) {
            accRe[ti][tj] = __builtin_amdgcn_mfma_f64_16x16x4f64(aRe[ti], bop[tj], accRe[ti][tj], 0, 0, 0);
            accIm[ti][tj] = __builtin_amdgcn_mfma_f64_16x16x4f64(aIm[ti], bop[tj], accIm[ti][tj], 0, 0, 0);
          }
      }
    }
  }
  if (!active) return;
  double2* out = reinterpret_cast<double2*>(partials) + (int64_t)blockIdx.x * In * In;
  for (int ti = 0; ti < 2; ++ti)
    for (int tj = 0; tj < 2; ++tj)
      for (int r = 0; r < 4; ++r) {
        const int i = si * kSuper + ri0 + ti * 16 + 4 * r + (lane >> 4);
        const int j = sj * kSuper + rj0 + tj * 16 + (lane & 15);
        if (i < In && j < In) out[(int64_t)i * In + j] = make_double2(accRe[ti][tj][r], accIm[ti][tj][r]);
      }
}

// gram[e] = sum over chunks of partials[chunk][e], in chunk order (deterministic).
__global__ void k_gram_reduce(const double* __restrict__ partials, int nchunks, int64_t n2,
                              double* __restrict__ gram) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n2) return;
  double acc = 0.;
  for (int c = 0; c < nchunks; ++c) acc += partials[(int64_t)c * n2 + e];
  gram[e] = acc;
}

// ---------------------------------------------------------------------------------------------
// Hermitian eigen-solve by parallel cyclic Jacobi (two-sided rotations, round-robin pairing).
// One workgroup per matrix; A and V live in global memory (L2-resident, <= 1 MiB each).
struct EigJob {
  const double* gram;   // n x n complex (interleaved), row-major
  double* A;            // work copy
  double* V;            // eigenvector accumulator
  float* U;             // out: n x r complex float32, row-major
  int n;
  int r;
};
struct EigJobs {
  EigJob job[kMaxNdim];
};

constexpr int kEigThreads = 1024;
constexpr int kEigMaxN = TGRAD_MAX_EXTENT;
constexpr int kEigMaxSweeps = 30;

__device__ __forceinline__ double2 cmuld(double2 a, double2 b) {
  return make_double2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ double2 conjd(double2 a) { return make_double2(a.x, -a.y); }

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

  for (int sweep = 0; sweep < kEigMaxSweeps; ++sweep) {
    if (tid == 0) nrot = 0;
    __syncthreads();
    for (int round = 0; round < m - 1; ++round) {
      // ---- phase 1: pairs of this round and their rotations ----
      if (tid < half) {
        int p, q;
        if (tid == 0) {
          p = m - 1;
          q = round;
        } else {
          p = (round + tid) % (m - 1);
          q = (round - tid + (m - 1)) % (m - 1);
        }
        if (p > q) {
          int t = p;
          p = q;
          q = t;
        }
        int rot = 0;
        double c = 1.;
        double2 s = make_double2(0., 0.);
        if (q < n) {                                   // q == n is the padding player of an odd n
          const double2 apq = A[p * n + q];
          const double app = A[p * n + p].x, aqq = A[q * n + q].x;
          const double mag2 = apq.x * apq.x + apq.y * apq.y;
          if (mag2 > eps2 * fabs(app * aqq) && mag2 > floor2) {
            const double mag = sqrt(mag2);
            const double tau = (aqq - app) / (2. * mag);
            const double t = (tau >= 0. ? 1. : -1.) / (fabs(tau) + sqrt(1. + tau * tau));
            c = 1. / sqrt(1. + t * t);
            const double sn = t * c;
            s = make_double2(sn * apq.x / mag, sn * apq.y / mag);   // s e^{i phi}
            rot = 1;
          }
        }
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
      for (int e = tid; e < 2 * n * half; e += kEigThreads) {
        const int which = e / (n * half);
        const int e2 = e - which * (n * half);
        const int i = e2 / half, pr = e2 - i * half;
        if (!srot[pr]) continue;
        double2* X = which ? V : A;
        const int p = sp[pr], q = sq[pr];
        const double c = sc[pr];
        const double2 s = ss[pr];
        const double2 xp = X[i * n + p], xq = X[i * n + q];
        const double2 t1 = cmuld(conjd(s), xq), t2 = cmuld(s, xp);
        X[i * n + p] = make_double2(c * xp.x - t1.x, c * xp.y - t1.y);
        X[i * n + q] = make_double2(t2.x + c * xq.x, t2.y + c * xq.y);
      }
      __syncthreads();
      // ---- phase 3: row rotations  A[p, :] <- c A[p, :] - s A[q, :],
      //                              A[q, :] <- conj(s) A[p, :] + c A[q, :] ----
      for (int e = tid; e < half * n; e += kEigThreads) {
        const int pr = e / n, j = e - pr * n;
        if (!srot[pr]) continue;
        const int p = sp[pr], q = sq[pr];
        const double c = sc[pr];
        const double2 s = ss[pr];
        const double2 xp = A[p * n + j], xq = A[q * n + j];
        const double2 t1 = cmuld(s, xq), t2 = cmuld(conjd(s), xp);
        A[p * n + j] = make_double2(c * xp.x - t1.x, c * xp.y - t1.y);
        A[q * n + j] = make_double2(t2.x + c * xq.x, t2.y + c * xq.y);
      }
      __syncthreads();
    }
    const int done = (nrot == 0);
    __syncthreads();
    if (done) break;
  }

  // ---- order eigenvalues descending (ties: lower index first), keep the first r ----
  for (int i = tid; i < n; i += kEigThreads) lam[i] = A[i * n + i].x;
  __syncthreads();
  for (int i = tid; i < n; i += kEigThreads) {
    int rank = 0;
    const double li = lam[i];
    for (int j = 0; j < n; ++j) rank += (lam[j] > li || (lam[j] == li && j < i)) ? 1 : 0;
    if (rank < r) col_of[rank] = i;
  }
  __syncthreads();
  // ---- unit phase per kept column: largest-modulus entry (first on ties) becomes real > 0 ----
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
  float2* U = reinterpret_cast<float2*>(jb.U);
  for (int e = tid; e < n * r; e += kEigThreads) {
    const int i = e / r, cidx = e - i * r;
    const double2 v = cmuld(V[i * n + col_of[cidx]], phase[cidx]);
    U[e] = make_float2((float)v.x, (float)v.y);
  }
}

__global__ void k_identity_factor(float2* U, int n) {
  int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n * n) U[e] = make_float2((e / n) == (e % n) ? 1.f : 0.f, 0.f);
}

}  // namespace

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
  dim3 grid((unsigned)nchunks, (unsigned)(nsup * nsup)), block(kGramThreads);
  if (dtype == TGRAD_C64)
    k_gram<TGRAD_C64><<<grid, block, 0, s>>>(g, mask, A, In, B, cols_per_chunk, partials);
  else
    k_gram<TGRAD_CBF16><<<grid, block, 0, s>>>(g, mask, A, In, B, cols_per_chunk, partials);
}

void launch_gram_reduce(hipStream_t s, const double* partials, int nchunks, int In, double* gram) {
  const int64_t n2 = (int64_t)In * In * 2;
  k_gram_reduce<<<dim3((unsigned)((n2 + 255) / 256)), dim3(256), 0, s>>>(partials, nchunks, n2, gram);
}

void launch_eig_batch(hipStream_t s, int njobs, const double* const* gram, double* const* work_a,
                      double* const* work_v, const int* In, const int* r, float* const* U) {
  if (njobs <= 0) return;
  EigJobs jobs;
  for (int i = 0; i < njobs; ++i) {
    jobs.job[i].gram = gram[i];
    jobs.job[i].A = work_a[i];
    jobs.job[i].V = work_v[i];
    jobs.job[i].U = U[i];
    jobs.job[i].n = In[i];
    jobs.job[i].r = r[i];
  }
  k_eig<<<dim3((unsigned)njobs), dim3(kEigThreads), 0, s>>>(jobs);
}

void launch_identity_factor(hipStream_t s, float* U, int n) {
  k_identity_factor<<<dim3((unsigned)((n * n + 255) / 256)), dim3(256), 0, s>>>(
      reinterpret_cast<float2*>(U), n);
}

}  // namespace tgrad
