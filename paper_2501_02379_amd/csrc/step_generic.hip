// Shape-generic kernels of the per-step path of Algorithm 1 (any ndim, any extents):
// gather of the sparse values, one mode-n product per launch, Adam on the Tucker core, the
// last reconstruction stage fused with the weight update, and Adam on the sparse values with
// the scatter-add into W.  One thread per output element; these are the reference-speed
// kernels every shape can use, and the fallback for shapes the MFMA kernels do not cover.
#include "device_common.h"

namespace tgrad {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float2 cmul(float2 u, float2 x) {          // u * x
  return make_float2(u.x * x.x - u.y * x.y, u.x * x.y + u.y * x.x);
}
__device__ __forceinline__ float2 cmul_conj(float2 u, float2 x) {     // conj(u) * x
  return make_float2(u.x * x.x + u.y * x.y, u.x * x.y - u.y * x.x);
}

// Sparse(G, Omega): values at the support, in Omega order (Algorithm 1, "Create sparse tensor
// at current step").
template <int DT>
__global__ void k_gather(const void* __restrict__ g, const int32_t* __restrict__ omega, int64_t k,
                         float2* __restrict__ out) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < k) out[j] = load_elem<DT>(g, omega[j]);
}

// Mode-n product (appendix "Tensor Operations and Notation", mode-k product), on the tensor
// viewed as (A, K, B):  out[a, m, b] = sum_k F[m, k] x[a, k, b].
//   PROJECT:  F = U^H  (F[m, k] = conj(U[k, m]), K = I_n, M = r_n)  - low-rank compression
//   !PROJECT: F = U    (F[m, k] = U[m, k],       K = r_n, M = I_n)  - reconstruction
// MASK: the input is the gradient itself and entries whose bit is set in `mask` (the support
// Omega) read as zero: this is G - Sparse(G, Omega) without materialising it.
template <int DT, bool MASK, bool PROJECT>
__global__ __launch_bounds__(kThreads) void k_contract(const void* __restrict__ x,
                                                       const uint32_t* __restrict__ mask,
                                                       const float2* __restrict__ U, int rn, int64_t A,
                                                       int K, int M, int64_t B,
                                                       float2* __restrict__ out) {
  const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (o >= A * M * B) return;
  const int64_t b = o % B;
  const int64_t am = o / B;
  const int m = (int)(am % M);
  const int64_t a = am / M;
  float2 acc = make_float2(0.f, 0.f);
  for (int k = 0; k < K; ++k) {
    const int64_t idx = (a * K + k) * B + b;
    if (MASK) {
      if ((mask[idx >> 5] >> (idx & 31)) & 1u) continue;
    }
    float2 v = load_elem<DT>(x, idx);
    float2 p = PROJECT ? cmul_conj(U[(int64_t)k * rn + m], v) : cmul(U[(int64_t)m * rn + k], v);
    acc.x += p.x;
    acc.y += p.y;
  }
  out[o] = acc;
}

// AdamUpdate on the compressed low-rank gradient (appendix algorithm "Adam with low-rank tensor
// decomposition": M, V from |R conj R|, bias correction, N = M^ / (sqrt(V^) + eps)).
__global__ void k_adam_core(const float2* __restrict__ r, float2* __restrict__ m, float* __restrict__ v,
                            float2* __restrict__ n_out, int64_t C, float beta1, float beta2,
                            float inv_c1, float inv_c2, float eps) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= C) return;
  float2 x = r[i];
  float2 mm = m[i];
  mm.x = beta1 * mm.x + (1.f - beta1) * x.x;
  mm.y = beta1 * mm.y + (1.f - beta1) * x.y;
  float vv = beta2 * v[i] + (1.f - beta2) * (x.x * x.x + x.y * x.y);
  m[i] = mm;
  v[i] = vv;
  float d = 1.f / (sqrtf(vv * inv_c2) + eps);
  n_out[i] = make_float2(mm.x * inv_c1 * d, mm.y * inv_c1 * d);
}

// AdamUpdate on the sparse values (appendix algorithm "Adam with low-rank tensor decomposition",
// applied to g_S): moments in place; gs[j] <- neg_lr_lambda * N_S[j], the scaled sparse update
// that k_update adds at Omega_j.
__global__ void k_sparse_adam(float2* __restrict__ gs, int64_t k, float2* __restrict__ m,
                              float* __restrict__ v, float beta1, float beta2, float inv_c1,
                              float inv_c2, float eps, float neg_lr_lambda) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= k) return;
  float2 x = gs[j];
  float2 mm = m[j];
  mm.x = beta1 * mm.x + (1.f - beta1) * x.x;
  mm.y = beta1 * mm.y + (1.f - beta1) * x.y;
  float vv = beta2 * v[j] + (1.f - beta2) * (x.x * x.x + x.y * x.y);
  m[j] = mm;
  v[j] = vv;
  float d = 1.f / (sqrtf(vv * inv_c2) + eps);
  gs[j] = make_float2(neg_lr_lambda * (mm.x * inv_c1 * d), neg_lr_lambda * (mm.y * inv_c1 * d));
}

__device__ __forceinline__ uint32_t bf16_bits_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Last reconstruction stage fused with the weight update (Algorithm 1, "Reconstruct low-rank
// part", "Add scaled sparse tensor" and W <- W + eta G~):
//   W[a, m] <- decay * W[a, m] + neg_lr_alpha * sum_k U[m, k] z[a, k]  (+ ns[j] where (a, m) = Omega_j).
// The support is found through the bitmask and a binary search of the ascending index list.
// WDT: weights stored as complex64, or as bf16 pairs that are widened, updated in float32 and
// rounded once to nearest even.
template <int WDT>
__global__ __launch_bounds__(kThreads) void k_update(const float2* __restrict__ z,
                                                     const float2* __restrict__ U, int rn, int64_t A,
                                                     int M, void* __restrict__ w, float decay,
                                                     float neg_lr_alpha, const uint32_t* __restrict__ mask,
                                                     const int32_t* __restrict__ omega, int64_t k,
                                                     const float2* __restrict__ ns) {
  const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (o >= A * M) return;
  const int m = (int)(o % M);
  const int64_t a = o / M;
  float2 acc = make_float2(0.f, 0.f);
  for (int kk = 0; kk < rn; ++kk) {
    float2 p = cmul(U[(int64_t)m * rn + kk], z[a * rn + kk]);
    acc.x += p.x;
    acc.y += p.y;
  }
  float2 upd = make_float2(neg_lr_alpha * acc.x, neg_lr_alpha * acc.y);
  if (mask && ((mask[o >> 5] >> (o & 31)) & 1u)) {
    int64_t lo = 0, hi = k - 1;                    // the bit is set, so o is in omega[0 .. k-1]
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if ((int64_t)omega[mid] < o) lo = mid + 1; else hi = mid;
    }
    const float2 sv = ns[lo];
    upd.x += sv.x;
    upd.y += sv.y;
  }
  if constexpr (WDT == TGRAD_C64) {
    float2* wp = reinterpret_cast<float2*>(w) + o;
    const float2 ww = *wp;
    *wp = make_float2(decay * ww.x + upd.x, decay * ww.y + upd.y);
  } else {
    uint32_t* wp = reinterpret_cast<uint32_t*>(w) + o;
    const uint32_t raw = *wp;
    const float re = decay * __uint_as_float(raw << 16) + upd.x;
    const float im = decay * __uint_as_float(raw & 0xFFFF0000u) + upd.y;
    *wp = bf16_bits_rne(re) | (bf16_bits_rne(im) << 16);
  }
}

// Residual of the low-rank approximation, R = G - G~_L (paragraph "Residual and composition"), from the
// tensor z = (G~_L before its last expansion), seen as (A, rn):  R[a, m] = G[a, m] - sum_k U[m, k] z[a, k].
//   k_residual        the whole tensor (refresh of the low-rank-first order: top-k runs on it);
//   k_residual_gather only at the support, in place on the gathered values: gs[j] <- gs[j] - G~_L[Omega_j].
template <int DT>
__global__ __launch_bounds__(kThreads) void k_residual(const void* __restrict__ g, const float2* __restrict__ z,
                                                       const float2* __restrict__ U, int rn, int64_t A, int M,
                                                       float2* __restrict__ r) {
  const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (o >= A * M) return;
  const int m = (int)(o % M);
  const int64_t a = o / M;
  float2 acc = make_float2(0.f, 0.f);
  for (int kk = 0; kk < rn; ++kk) {
    float2 p = cmul(U[(int64_t)m * rn + kk], z[a * rn + kk]);
    acc.x += p.x;
    acc.y += p.y;
  }
  const float2 gv = load_elem<DT>(g, o);
  r[o] = make_float2(gv.x - acc.x, gv.y - acc.y);
}

__global__ void k_residual_gather(float2* __restrict__ gs, const int32_t* __restrict__ omega, int64_t k,
                                  const float2* __restrict__ z, const float2* __restrict__ U, int rn, int M) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= k) return;
  const int64_t o = omega[j];
  const int m = (int)(o % M);
  const int64_t a = o / M;
  float2 acc = make_float2(0.f, 0.f);
  for (int kk = 0; kk < rn; ++kk) {
    float2 p = cmul(U[(int64_t)m * rn + kk], z[a * rn + kk]);
    acc.x += p.x;
    acc.y += p.y;
  }
  const float2 gv = gs[j];
  gs[j] = make_float2(gv.x - acc.x, gv.y - acc.y);
}

inline unsigned blocks_for(int64_t n, int threads) { return (unsigned)((n + threads - 1) / threads); }

}  // namespace

void launch_gather(hipStream_t s, const void* g, int dtype, const int32_t* omega, int64_t k, float2* out) {
  if (k <= 0) return;
  if (dtype == TGRAD_C64)
    k_gather<TGRAD_C64><<<dim3(blocks_for(k, 256)), dim3(256), 0, s>>>(g, omega, k, out);
  else
    k_gather<TGRAD_CBF16><<<dim3(blocks_for(k, 256)), dim3(256), 0, s>>>(g, omega, k, out);
}

void launch_contract(hipStream_t s, const void* x, int x_dtype, const uint32_t* mask, const float2* U,
                     int In, int rn, bool project, const Stage& st, float2* out) {
  (void)In;
  const int64_t total = st.A * st.M * st.B;
  if (total <= 0) return;
  dim3 grid(blocks_for(total, kThreads)), block(kThreads);
#define TGRAD_GO(DT, MASK, PROJ) \
  k_contract<DT, MASK, PROJ><<<grid, block, 0, s>>>(x, mask, U, rn, st.A, st.K, st.M, st.B, out)
  if (x_dtype == TGRAD_CBF16) {
    if (mask) TGRAD_GO(TGRAD_CBF16, true, true); else TGRAD_GO(TGRAD_CBF16, false, true);
  } else if (project) {
    if (mask) TGRAD_GO(TGRAD_C64, true, true); else TGRAD_GO(TGRAD_C64, false, true);
  } else {
    TGRAD_GO(TGRAD_C64, false, false);
  }
#undef TGRAD_GO
}

void launch_adam_core(hipStream_t s, const float2* r, float2* m, float* v, float2* n_out, int64_t C,
                      float beta1, float beta2, float inv_c1, float inv_c2, float eps) {
  k_adam_core<<<dim3(blocks_for(C, 256)), dim3(256), 0, s>>>(r, m, v, n_out, C, beta1, beta2, inv_c1,
                                                            inv_c2, eps);
}

void launch_sparse_adam(hipStream_t s, float2* gs, int64_t k, float2* m, float* v, float beta1, float beta2,
                        float inv_c1, float inv_c2, float eps, float neg_lr_lambda) {
  if (k <= 0) return;
  k_sparse_adam<<<dim3(blocks_for(k, 256)), dim3(256), 0, s>>>(gs, k, m, v, beta1, beta2, inv_c1, inv_c2, eps,
                                                              neg_lr_lambda);
}

void launch_update(hipStream_t s, const float2* z, const float2* U, int In, int rn, const Stage& st, void* w,
                   int wdtype, float decay, float neg_lr_alpha, const uint32_t* mask, const int32_t* omega,
                   int64_t k, const float2* ns) {
  (void)In;
  const int64_t total = st.A * st.M;
  if (total <= 0) return;
  dim3 grid(blocks_for(total, kThreads)), block(kThreads);
  if (wdtype == TGRAD_C64)
    k_update<TGRAD_C64><<<grid, block, 0, s>>>(z, U, rn, st.A, st.M, w, decay, neg_lr_alpha, mask, omega, k, ns);
  else
    k_update<TGRAD_CBF16><<<grid, block, 0, s>>>(z, U, rn, st.A, st.M, w, decay, neg_lr_alpha, mask, omega, k, ns);
}

void launch_residual(hipStream_t s, const void* g, int dtype, const float2* z, const float2* U, int rn, int64_t A,
                     int M, float2* r) {
  const int64_t total = A * M;
  if (total <= 0) return;
  dim3 grid(blocks_for(total, kThreads)), block(kThreads);
  if (dtype == TGRAD_C64)
    k_residual<TGRAD_C64><<<grid, block, 0, s>>>(g, z, U, rn, A, M, r);
  else
    k_residual<TGRAD_CBF16><<<grid, block, 0, s>>>(g, z, U, rn, A, M, r);
}

void launch_residual_gather(hipStream_t s, float2* gs, const int32_t* omega, int64_t k, const float2* z,
                            const float2* U, int rn, int M) {
  if (k <= 0) return;
  k_residual_gather<<<dim3(blocks_for(k, 256)), dim3(256), 0, s>>>(gs, omega, k, z, U, rn, M);
}

}  // namespace tgrad
