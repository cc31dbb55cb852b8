// Sparse-support selection: Omega <- SparseIndices(G, rho, top-k magnitude), the first line of
// the refresh branch of Algorithm 1 (and section "Unstructured sparse gradient tensor":
// k = ceil(rho I) entries, kept as index/value pairs).
//
// Order: (|g|^2 descending, linear index ascending); Omega is written ascending.
//
// Method: most-significant-digit radix select on the 32-bit pattern of the float32 key
// (digits of 12, 12 and 8 bits -> three histogram passes), which yields the key T of the k-th
// largest entry and the number `need_eq` of entries equal to T that belong to the support (the
// ones with the lowest indices).  A count pass and an emit pass then place every selected entry:
// the position of entry i inside Omega is
//     #(key > T before i) + min(#(key == T before i), need_eq),
// so two independent exclusive prefix counts are enough and no atomics decide an output slot.
// Everything is integer work: the result is bit-exact and run-to-run deterministic.
//
// Uniform random selection (rand-k, the alternative rule the same section names) runs through the
// same passes with a different key: key(i) = fmix32(fmix32(i xor s0) + s1), fmix32 the 32-bit
// finalizer of MurmurHash3 and (s0, s1) two words made from the seed and the step count of the
// refresh.  The key map is a bijection, so no two entries tie, and the gradient is never read.
#include "device_common.h"

namespace tgrad {

namespace {

constexpr int kSelThreads = 256;
constexpr int kWavesPerBlock = kSelThreads / kWave;
constexpr int kPairsPerIter = kWave;                       // one pair (2 elements) per lane
constexpr int kSegIters = kSegElems / (2 * kPairsPerIter); // 16 iterations of 128 elements

__device__ __forceinline__ uint32_t digit_of(uint32_t key, int pass) {
  return pass == 0 ? (key >> 20) : pass == 1 ? ((key >> 8) & 0xFFFu) : (key & 0xFFu);
}
__device__ __forceinline__ bool in_prefix(uint32_t key, int pass, uint32_t prefix) {
  return pass == 0 ? true : pass == 1 ? ((key >> 20) == prefix) : ((key >> 8) == prefix);
}

// Where the keys come from: the gradient (KS = its dtype) or the index hash (KS = kKeyRandom).
constexpr int kKeyRandom = 2;
struct KeySource {
  const void* g;
  uint32_t s0, s1;
};

__device__ __forceinline__ uint32_t fmix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x85EBCA6Bu;
  x ^= x >> 13;
  x *= 0xC2B2AE35u;
  x ^= x >> 16;
  return x;
}

// Keys of elements 2p and 2p+1 (the caller guarantees 2p + 1 < I).
template <int KS>
__device__ __forceinline__ void pair_keys(const KeySource& src, int64_t p, uint32_t& k0, uint32_t& k1) {
  if constexpr (KS == kKeyRandom) {
    const uint32_t i0 = (uint32_t)(2 * p);
    k0 = fmix32(fmix32(i0 ^ src.s0) + src.s1);
    k1 = fmix32(fmix32((i0 + 1u) ^ src.s0) + src.s1);
  } else {
    float2 e0, e1;
    load_pair<KS>(src.g, p, e0, e1);
    k0 = select_key(e0);
    k1 = select_key(e1);
  }
}
template <int KS>
__device__ __forceinline__ uint32_t elem_key(const KeySource& src, int64_t i) {
  if constexpr (KS == kKeyRandom)
    return fmix32(fmix32((uint32_t)i ^ src.s0) + src.s1);
  else
    return select_key(load_elem<KS>(src.g, i));
}

template <int DT>
__global__ __launch_bounds__(kSelThreads) void k_select_hist(const KeySource g, int64_t I,
                                                             int pass,
                                                             const SelectScalars* __restrict__ sc,
                                                             uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[kHistBins];
  for (int b = threadIdx.x; b < kHistBins; b += kSelThreads) h[b] = 0;
  __syncthreads();
  const uint32_t prefix = pass == 0 ? 0u : sc->prefix;
  const int64_t npairs = I >> 1;
  const int64_t stride = (int64_t)gridDim.x * kSelThreads;
  for (int64_t p = (int64_t)blockIdx.x * kSelThreads + threadIdx.x; p < npairs; p += stride) {
    uint32_t k0, k1;
    pair_keys<DT>(g, p, k0, k1);
    if (in_prefix(k0, pass, prefix)) atomicAdd(&h[digit_of(k0, pass)], 1u);
    if (in_prefix(k1, pass, prefix)) atomicAdd(&h[digit_of(k1, pass)], 1u);
  }
  if ((I & 1) && blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t k0 = elem_key<DT>(g, I - 1);
    if (in_prefix(k0, pass, prefix)) atomicAdd(&h[digit_of(k0, pass)], 1u);
  }
  __syncthreads();
  for (int b = threadIdx.x; b < kHistBins; b += kSelThreads)
    if (h[b]) atomicAdd(&hist[b], h[b]);
}

// One block of 1024 threads: find the digit bin that holds the `remaining`-th largest entry.
__global__ __launch_bounds__(1024) void k_select_pick(int pass, uint32_t k, SelectScalars* sc,
                                                      const uint32_t* __restrict__ hist) {
  __shared__ uint32_t scan[1024];
  const int t = threadIdx.x;
  uint32_t c[4];
  uint32_t local = 0;
  for (int b = 0; b < 4; ++b) {
    c[b] = hist[4 * t + b];
    local += c[b];
  }
  // inclusive scan over threads in DESCENDING bin order: slot j holds thread 1023 - j
  scan[1023 - t] = local;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    uint32_t v = scan[t];
    uint32_t add = t >= off ? scan[t - off] : 0u;
    __syncthreads();
    scan[t] = v + add;
    __syncthreads();
  }
  uint32_t above = scan[1023 - t] - local;           // entries in bins owned by higher threads
  const uint32_t rem = pass == 0 ? k : sc->remaining;
  const uint32_t prefix = pass == 0 ? 0u : sc->prefix;
  __syncthreads();                                    // everyone has read sc before one thread writes
  for (int b = 3; b >= 0; --b) {
    if (above < rem && rem <= above + c[b]) {
      uint32_t bin = 4u * t + b;
      uint32_t np = pass == 0 ? bin : pass == 1 ? ((prefix << 12) | bin) : ((prefix << 8) | bin);
      sc->prefix = np;
      sc->remaining = rem - above;
      if (pass == 2) {
        sc->threshold = np;
        sc->need_eq = rem - above;
      }
    }
    above += c[b];
  }
}

// Flags of the (up to) two elements a lane holds in iteration `it` of segment `seg`.
template <int DT>
__device__ __forceinline__ void seg_keys(const KeySource& g, int64_t I, int64_t seg, int it, int lane,
                                         int64_t& i0, bool& v0, bool& v1, uint32_t& k0, uint32_t& k1) {
  i0 = seg * kSegElems + (int64_t)it * (2 * kPairsPerIter) + 2 * lane;
  v0 = i0 < I;
  v1 = i0 + 1 < I;
  k0 = 0;
  k1 = 0;
  if (v1) {
    pair_keys<DT>(g, i0 >> 1, k0, k1);
  } else if (v0) {
    k0 = elem_key<DT>(g, i0);
  }
}

template <int DT>
__global__ __launch_bounds__(kSelThreads) void k_select_count(const KeySource g, int64_t I,
                                                              const SelectScalars* __restrict__ sc,
                                                              uint32_t* __restrict__ seg_gt,
                                                              uint32_t* __restrict__ seg_eq,
                                                              int64_t nseg) {
  const int lane = lane_id();
  const int64_t seg = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
  if (seg >= nseg) return;                           // whole wave leaves together
  const uint32_t T = sc->threshold;
  uint32_t ngt = 0, neq = 0;
  for (int it = 0; it < kSegIters; ++it) {
    int64_t i0;
    bool v0, v1;
    uint32_t k0, k1;
    seg_keys<DT>(g, I, seg, it, lane, i0, v0, v1, k0, k1);
    ngt += __popcll(__ballot(v0 && k0 > T)) + __popcll(__ballot(v1 && k1 > T));
    neq += __popcll(__ballot(v0 && k0 == T)) + __popcll(__ballot(v1 && k1 == T));
  }
  if (lane == 0) {
    seg_gt[seg] = ngt;
    seg_eq[seg] = neq;
  }
}

// In-place exclusive prefix sums of both per-segment count arrays; one block of 16 wavefronts.
// Wavefront w owns the contiguous range [w * per, (w + 1) * per): it first adds the range up
// (coalesced 64-entry reads), the 16 totals are scanned through LDS, then the range is walked again
// and every 64-entry group is scanned with lane shuffles on top of the running offset.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int lane) {
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint32_t up = __shfl_up(v, off, kWave);
    if (lane >= off) v += up;
  }
  return v;
}

__global__ __launch_bounds__(1024) void k_select_scan(uint32_t* seg_gt, uint32_t* seg_eq, int64_t nseg) {
  __shared__ uint32_t tot_g[16], tot_e[16];
  const int lane = lane_id();
  const int wave = threadIdx.x / kWave;
  const int64_t per = ((nseg + 15) / 16 + kWave - 1) / kWave * kWave;       // a multiple of the group size
  const int64_t lo = wave * per;
  const int64_t hi = lo + per < nseg ? lo + per : nseg;
  uint32_t a = 0, b = 0;
  for (int64_t i = lo + lane; i < hi; i += kWave) {
    a += seg_gt[i];
    b += seg_eq[i];
  }
  a = wave_inclusive_scan(a, lane);
  b = wave_inclusive_scan(b, lane);
  if (lane == kWave - 1) {
    tot_g[wave] = a;
    tot_e[wave] = b;
  }
  __syncthreads();
  uint32_t run_g = 0, run_e = 0;                      // entries in the ranges of lower wavefronts
  for (int w = 0; w < wave; ++w) {
    run_g += tot_g[w];
    run_e += tot_e[w];
  }
  for (int64_t i0 = lo; i0 < hi; i0 += kWave) {
    const int64_t i = i0 + lane;
    const uint32_t cg = i < hi ? seg_gt[i] : 0u, ce = i < hi ? seg_eq[i] : 0u;
    const uint32_t sg = wave_inclusive_scan(cg, lane), se = wave_inclusive_scan(ce, lane);
    if (i < hi) {
      seg_gt[i] = run_g + sg - cg;
      seg_eq[i] = run_e + se - ce;
    }
    run_g += __shfl(sg, kWave - 1, kWave);
    run_e += __shfl(se, kWave - 1, kWave);
  }
}

// Spread the low 16 bits of x to the even bit positions of a 32-bit word.
__device__ __forceinline__ uint32_t spread16(uint32_t x) {
  x &= 0xFFFFu;
  x = (x | (x << 8)) & 0x00FF00FFu;
  x = (x | (x << 4)) & 0x0F0F0F0Fu;
  x = (x | (x << 2)) & 0x33333333u;
  x = (x | (x << 1)) & 0x55555555u;
  return x;
}

template <int DT>
__global__ __launch_bounds__(kSelThreads) void k_select_emit(const KeySource g, int64_t I,
                                                             const SelectScalars* __restrict__ sc,
                                                             const uint32_t* __restrict__ seg_gt,
                                                             const uint32_t* __restrict__ seg_eq,
                                                             int64_t nseg, int32_t* __restrict__ omega,
                                                             uint32_t* __restrict__ mask) {
  const int lane = lane_id();
  const int64_t seg = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
  if (seg >= nseg) return;
  const uint32_t T = sc->threshold;
  const uint32_t need = sc->need_eq;
  uint32_t run_gt = seg_gt[seg], run_eq = seg_eq[seg];
  for (int it = 0; it < kSegIters; ++it) {
    int64_t i0;
    bool v0, v1;
    uint32_t k0, k1;
    seg_keys<DT>(g, I, seg, it, lane, i0, v0, v1, k0, k1);
    const bool g0 = v0 && k0 > T, g1 = v1 && k1 > T;
    const bool e0 = v0 && k0 == T, e1 = v1 && k1 == T;
    const uint64_t Bg0 = __ballot(g0), Bg1 = __ballot(g1), Be0 = __ballot(e0), Be1 = __ballot(e1);
    // entries before element i0 (in index order: lower lanes hold lower indices)
    uint32_t gtb = run_gt + popc_below(Bg0, lane) + popc_below(Bg1, lane);
    uint32_t eqb = run_eq + popc_below(Be0, lane) + popc_below(Be1, lane);
    bool s0 = false, s1 = false;
    if (g0) {
      s0 = true;
      omega[gtb + (eqb < need ? eqb : need)] = (int32_t)i0;
    } else if (e0 && eqb < need) {
      s0 = true;
      omega[gtb + eqb] = (int32_t)i0;
    }
    gtb += g0 ? 1u : 0u;                               // element i0 + 1 comes after element i0
    eqb += e0 ? 1u : 0u;
    if (g1) {
      s1 = true;
      omega[gtb + (eqb < need ? eqb : need)] = (int32_t)(i0 + 1);
    } else if (e1 && eqb < need) {
      s1 = true;
      omega[gtb + eqb] = (int32_t)(i0 + 1);
    }
    const uint64_t S0 = __ballot(s0), S1 = __ballot(s1);
    if ((lane & 15) == 0 && i0 < I) {
      uint32_t w = spread16((uint32_t)(S0 >> lane)) | (spread16((uint32_t)(S1 >> lane)) << 1);
      mask[i0 >> 5] = w;
    }
    run_gt += __popcll(Bg0) + __popcll(Bg1);
    run_eq += __popcll(Be0) + __popcll(Be1);
  }
}

__global__ void k_mask_from_indices(const int32_t* __restrict__ omega, int64_t k, uint32_t* mask) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < k) {
    uint32_t i = (uint32_t)omega[j];
    atomicOr(&mask[i >> 5], 1u << (i & 31));
  }
}

// Plain streaming copy (16 bytes per lane per step), the reference point for memory counters.
__global__ __launch_bounds__(256) void k_copy16(float4* __restrict__ dst, const float4* __restrict__ src,
                                                int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ void k_zero_u32(uint32_t* p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

}  // namespace

void launch_copy16(hipStream_t s, void* dst, const void* src, int64_t n16) {
  if (n16 <= 0) return;
  const int64_t want = (n16 + 255) / 256;
  const unsigned grid = (unsigned)(want < 256 * 16 ? want : 256 * 16);
  k_copy16<<<dim3(grid), dim3(256), 0, s>>>(reinterpret_cast<float4*>(dst), reinterpret_cast<const float4*>(src),
                                            n16);
}

void zero_u32(hipStream_t s, uint32_t* p, int64_t n) {
  if (n <= 0) return;
  k_zero_u32<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(p, n);
}

void launch_select_hist(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                        int pass, const SelectScalars* sc, uint32_t* hist) {
  int64_t npairs = I >> 1;
  int64_t want = (npairs + kSelThreads - 1) / kSelThreads;
  unsigned grid = (unsigned)(want < 1 ? 1 : want > 4096 ? 4096 : want);
  const KeySource src{g, keys.s0, keys.s1};
  if (keys.random)
    k_select_hist<kKeyRandom><<<dim3(grid), dim3(kSelThreads), 0, s>>>(src, I, pass, sc, hist);
  else if (dtype == TGRAD_C64)
    k_select_hist<TGRAD_C64><<<dim3(grid), dim3(kSelThreads), 0, s>>>(src, I, pass, sc, hist);
  else
    k_select_hist<TGRAD_CBF16><<<dim3(grid), dim3(kSelThreads), 0, s>>>(src, I, pass, sc, hist);
}

void launch_select_pick(hipStream_t s, int pass, uint32_t k, SelectScalars* sc, const uint32_t* hist) {
  k_select_pick<<<dim3(1), dim3(1024), 0, s>>>(pass, k, sc, hist);
}

void launch_select_count(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                         const SelectScalars* sc, uint32_t* seg_gt, uint32_t* seg_eq, int64_t nseg) {
  unsigned grid = (unsigned)((nseg + kWavesPerBlock - 1) / kWavesPerBlock);
  const KeySource src{g, keys.s0, keys.s1};
  if (keys.random)
    k_select_count<kKeyRandom><<<dim3(grid), dim3(kSelThreads), 0, s>>>(src, I, sc, seg_gt, seg_eq, nseg);
  else if (dtype == TGRAD_C64)
    k_select_count<TGRAD_C64><<<dim3(grid), dim3(kSelThreads), 0, s>>>(src, I, sc, seg_gt, seg_eq, nseg);
  else
    k_select_count<TGRAD_CBF16><<<dim3(grid), dim3(kSelThreads), 0, s>>>(src, I, sc, seg_gt, seg_eq, nseg);
}

void launch_select_scan(hipStream_t s, uint32_t* seg_gt, uint32_t* seg_eq, int64_t nseg) {
  k_select_scan<<<dim3(1), dim3(1024), 0, s>>>(seg_gt, seg_eq, nseg);
}

void launch_select_emit(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                        const SelectScalars* sc, const uint32_t* seg_gt, const uint32_t* seg_eq,
                        int64_t nseg, int32_t* omega, uint32_t* mask) {
  unsigned grid = (unsigned)((nseg + kWavesPerBlock - 1) / kWavesPerBlock);
  const KeySource src{g, keys.s0, keys.s1};
  if (keys.random)
    k_select_emit<kKeyRandom><<<dim3(grid), dim3(kSelThreads), 0, s>>>(src, I, sc, seg_gt, seg_eq, nseg,
                                                                       omega, mask);
  else if (dtype == TGRAD_C64)
    k_select_emit<TGRAD_C64><<<dim3(grid), dim3(kSelThreads), 0, s>>>(src, I, sc, seg_gt, seg_eq, nseg,
                                                                      omega, mask);
  else
    k_select_emit<TGRAD_CBF16><<<dim3(grid), dim3(kSelThreads), 0, s>>>(src, I, sc, seg_gt, seg_eq, nseg,
                                                                        omega, mask);
}

void launch_mask_from_indices(hipStream_t s, const int32_t* omega, int64_t k, uint32_t* mask,
                              int64_t mask_words) {
  zero_u32(s, mask, mask_words);
  if (k > 0)
    k_mask_from_indices<<<dim3((unsigned)((k + 255) / 256)), dim3(256), 0, s>>>(omega, k, mask);
}

}  // namespace tgrad
