// Sparse-support selection: Omega <- SparseIndices(G, rho, top-k magnitude), the first line of
// the refresh branch of Algorithm 1 (and section "Unstructured sparse gradient tensor":
// k = ceil(rho I) entries, kept as index/value pairs).
//
// Order: (|g|^2 descending, linear index ascending); Omega is written ascending.
//
// Method: most-significant-digit radix select on the 32-bit pattern of the float32 key (digits of
// 12, 12 and 8 bits), arranged so that the gradient is streamed only TWICE:
//   1. k_select_hist    reads G: histogram of the leading 12 key bits -> the bin b1 that holds the
//                       k-th largest key.
//   2. k_select_split   reads G: one bit per element into two bitmasks: "sure" (leading digit above
//                       b1: certainly in the support) and "cand" (leading digit equal to b1: the
//                       candidates among which the remaining digits decide).
//   3. k_select_hist_cand (twice) walks the candidate mask and fetches only the candidates' keys:
//                       histograms of the middle 12 and the last 8 bits -> the key T of the k-th
//                       largest entry and the number `need_eq` of entries equal to T that belong to
//                       the support (the ones with the lowest indices).
//   4. k_select_count / k_select_scan / k_select_emit walk the two masks (and the candidates' keys):
//                       the position of entry i inside Omega is
//                           #(key > T before i) + min(#(key == T before i), need_eq),
//                       two exclusive prefix counts, so no atomics decide an output slot.  The emit
//                       kernel also turns the "sure" mask into the support bitmask.
// The candidates are the entries of ONE of 4096 key bins (16 per octave of |g|^2), a fraction of a
// percent of the tensor for any smooth distribution; on a degenerate input (all keys equal) every
// element is a candidate and steps 3 and 4 read all of G through the same code, only slower.
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
constexpr int kChunkWords = kSelChunkElems / 32;           // mask words one wavefront counts / emits in order

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

// Histogram of the leading 12 key bits of every element.
template <int DT>
__global__ __launch_bounds__(kSelThreads) void k_select_hist(const KeySource g, int64_t I,
                                                             uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[kHistBins];
  for (int b = threadIdx.x; b < kHistBins; b += kSelThreads) h[b] = 0;
  __syncthreads();
  const int64_t npairs = I >> 1;
  const int64_t stride = (int64_t)gridDim.x * kSelThreads;
  for (int64_t p = (int64_t)blockIdx.x * kSelThreads + threadIdx.x; p < npairs; p += stride) {
    uint32_t k0, k1;
    pair_keys<DT>(g, p, k0, k1);
    atomicAdd(&h[digit_of(k0, 0)], 1u);
    atomicAdd(&h[digit_of(k1, 0)], 1u);
  }
  if ((I & 1) && blockIdx.x == 0 && threadIdx.x == 0) atomicAdd(&h[digit_of(elem_key<DT>(g, I - 1), 0)], 1u);
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

// Keys of the (up to) two elements a lane holds in iteration `it` of segment `seg`.
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

// Spread the low 16 bits of x to the even bit positions of a 32-bit word.
__device__ __forceinline__ uint32_t spread16(uint32_t x) {
  x &= 0xFFFFu;
  x = (x | (x << 8)) & 0x00FF00FFu;
  x = (x | (x << 4)) & 0x0F0F0F0Fu;
  x = (x | (x << 2)) & 0x33333333u;
  x = (x | (x << 1)) & 0x55555555u;
  return x;
}

// One bit per element into the two masks (bit b of word w = element 32 w + b): `sure` where the
// leading key digit lies above the bin b1 of the first pick, `cand` where it equals b1.  Bits past
// the end of the tensor are written as zero; every word that covers an element is written.
template <int DT>
__global__ __launch_bounds__(kSelThreads) void k_select_split(const KeySource g, int64_t I,
                                                              const SelectScalars* __restrict__ sc,
                                                              uint32_t* __restrict__ sure,
                                                              uint32_t* __restrict__ cand, int64_t nseg) {
  const int lane = lane_id();
  const int64_t seg = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
  if (seg >= nseg) return;                           // whole wave leaves together
  const uint32_t b1 = sc->prefix;                    // after the first pick: the leading digit of T
  for (int it = 0; it < kSegIters; ++it) {
    int64_t i0;
    bool v0, v1;
    uint32_t k0, k1;
    seg_keys<DT>(g, I, seg, it, lane, i0, v0, v1, k0, k1);
    const uint32_t d0 = k0 >> 20, d1 = k1 >> 20;
    const uint64_t S0 = __ballot(v0 && d0 > b1), S1 = __ballot(v1 && d1 > b1);
    const uint64_t C0 = __ballot(v0 && d0 == b1), C1 = __ballot(v1 && d1 == b1);
    if ((lane & 15) == 0 && i0 < I) {
      sure[i0 >> 5] = spread16((uint32_t)(S0 >> lane)) | (spread16((uint32_t)(S1 >> lane)) << 1);
      cand[i0 >> 5] = spread16((uint32_t)(C0 >> lane)) | (spread16((uint32_t)(C1 >> lane)) << 1);
    }
  }
}

// Histogram of the next digit over the candidates only (pass 1: bits 19..8 of the keys whose
// leading digit is the picked one - every candidate; pass 2: bits 7..0 of the keys whose leading
// 24 bits are the picked ones).  A lane owns one mask word per iteration and fetches the keys of
// its set bits.
template <int DT>
__global__ __launch_bounds__(kSelThreads) void k_select_hist_cand(const KeySource g, int pass,
                                                                  const SelectScalars* __restrict__ sc,
                                                                  const uint32_t* __restrict__ cand,
                                                                  int64_t nwords, uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[kHistBins];
  for (int b = threadIdx.x; b < kHistBins; b += kSelThreads) h[b] = 0;
  __syncthreads();
  const uint32_t prefix = sc->prefix;
  const int64_t stride = (int64_t)gridDim.x * kSelThreads;
  for (int64_t w = (int64_t)blockIdx.x * kSelThreads + threadIdx.x; w < nwords; w += stride) {
    uint32_t c = cand[w];
    while (c) {
      const int b = __builtin_ctz(c);
      c &= c - 1u;
      const uint32_t key = elem_key<DT>(g, (w << 5) + b);
      if (in_prefix(key, pass, prefix)) atomicAdd(&h[digit_of(key, pass)], 1u);
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < kHistBins; b += kSelThreads)
    if (h[b]) atomicAdd(&hist[b], h[b]);
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// Candidate bits of one mask word sorted by their key against the threshold T.
template <int DT>
__device__ __forceinline__ void classify_candidates(const KeySource& g, int64_t w, uint32_t c, uint32_t T,
                                                    uint32_t& above, uint32_t& equal) {
  above = 0u;
  equal = 0u;
  while (c) {
    const int b = __builtin_ctz(c);
    c &= c - 1u;
    const uint32_t key = elem_key<DT>(g, (w << 5) + b);
    if (key > T) above |= 1u << b;
    else if (key == T) equal |= 1u << b;
  }
}

// Per chunk of kChunkWords mask words (one wavefront each): entries above T and entries equal to T.
template <int DT>
__global__ __launch_bounds__(kSelThreads) void k_select_count(const KeySource g,
                                                              const SelectScalars* __restrict__ sc,
                                                              const uint32_t* __restrict__ sure,
                                                              const uint32_t* __restrict__ cand, int64_t nwords,
                                                              uint32_t* __restrict__ chunk_gt,
                                                              uint32_t* __restrict__ chunk_eq, int64_t nchunks) {
  const int lane = lane_id();
  const int64_t chunk = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
  if (chunk >= nchunks) return;
  const uint32_t T = sc->threshold;
  uint32_t ngt = 0, neq = 0;
  for (int it = 0; it < kChunkWords / kWave; ++it) {
    const int64_t w = chunk * kChunkWords + (int64_t)it * kWave + lane;
    if (w < nwords) {
      uint32_t above, equal;
      classify_candidates<DT>(g, w, cand[w], T, above, equal);
      ngt += __popc(sure[w]) + __popc(above);
      neq += __popc(equal);
    }
  }
  ngt = wave_sum(ngt);
  neq = wave_sum(neq);
  if (lane == 0) {
    chunk_gt[chunk] = ngt;
    chunk_eq[chunk] = neq;
  }
}

// In-place exclusive prefix sums of both per-chunk count arrays; one block of 16 wavefronts.
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

// Ordered compaction: a wavefront walks its chunk of mask words in index order (lane = word inside
// a group of 64, bits ascending inside a word) and writes every selected index to its final slot.
// `sure` comes in as the mask of the entries whose leading digit lies above the picked bin and goes
// out as the support bitmask (those, the candidates above T and the first need_eq candidates equal
// to T).
template <int DT>
__global__ __launch_bounds__(kSelThreads) void k_select_emit(const KeySource g,
                                                             const SelectScalars* __restrict__ sc,
                                                             const uint32_t* __restrict__ chunk_gt,
                                                             const uint32_t* __restrict__ chunk_eq,
                                                             int64_t nchunks, uint32_t* __restrict__ sure,
                                                             const uint32_t* __restrict__ cand, int64_t nwords,
                                                             int32_t* __restrict__ omega) {
  const int lane = lane_id();
  const int64_t chunk = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x / kWave);
  if (chunk >= nchunks) return;
  const uint32_t T = sc->threshold;
  const uint32_t need = sc->need_eq;
  uint32_t run_gt = chunk_gt[chunk], run_eq = chunk_eq[chunk];
  for (int it = 0; it < kChunkWords / kWave; ++it) {
    const int64_t w = chunk * kChunkWords + (int64_t)it * kWave + lane;
    uint32_t take = 0u, equal = 0u;                   // bits taken for certain; bits equal to T
    if (w < nwords) {
      uint32_t above;
      classify_candidates<DT>(g, w, cand[w], T, above, equal);
      take = sure[w] | above;
    }
    const uint32_t ng = __popc(take), ne = __popc(equal);
    const uint32_t sg = wave_inclusive_scan(ng, lane), se = wave_inclusive_scan(ne, lane);
    uint32_t gtb = run_gt + sg - ng, eqb = run_eq + se - ne;   // entries before this word
    uint32_t todo = take | equal, chosen = take;
    while (todo) {
      const int b = __builtin_ctz(todo);
      todo &= todo - 1u;
      const int32_t idx = (int32_t)((w << 5) + b);
      if (take & (1u << b)) {
        omega[gtb + (eqb < need ? eqb : need)] = idx;
        ++gtb;
      } else {
        if (eqb < need) {
          omega[gtb + eqb] = idx;
          chosen |= 1u << b;
        }
        ++eqb;
      }
    }
    if (w < nwords) sure[w] = chosen;
    run_gt += __shfl(sg, kWave - 1, kWave);
    run_eq += __shfl(se, kWave - 1, kWave);
  }
}

__global__ void k_mask_from_indices(const int32_t* __restrict__ omega, int64_t k, uint32_t* mask) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < k) {
    uint32_t i = (uint32_t)omega[j];
    atomicOr(&mask[i >> 5], 1u << (i & 31));
  }
}

// Plain streaming copy, the reference point for memory counters and for the copy rate this box
// reaches: every lane keeps four 16-byte pieces in flight (the same depth the optimizer's streaming
// kernels use), loads and stores marked non-temporal like theirs.
typedef float f32x4c __attribute__((ext_vector_type(4)));
constexpr int kCopyDepth = 4;
__global__ __launch_bounds__(256) void k_copy16(f32x4c* __restrict__ dst, const f32x4c* __restrict__ src,
                                                int64_t n16) {
  // a workgroup moves contiguous runs of 256 * kCopyDepth pieces (16 KB), run after run
  constexpr int64_t kRun = 256 * kCopyDepth;
  const int64_t nruns = n16 / kRun;
  for (int64_t r = blockIdx.x; r < nruns; r += gridDim.x) {
    const int64_t base = r * kRun + threadIdx.x;
    f32x4c v[kCopyDepth];
#pragma unroll
    for (int u = 0; u < kCopyDepth; ++u) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
    for (int u = 0; u < kCopyDepth; ++u) __builtin_nontemporal_store(v[u], dst + base + u * 256);
  }
  for (int64_t i = nruns * kRun + (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// The access pattern of the weight-update kernel without its arithmetic: a wavefront owns a tile of
// `tile_pieces` 16-byte pieces (at most kTilePieces x 64), loads all of it, then stores all of it back in
// place; wavefronts take slabs of `S` consecutive tiles, slabs dealt round-robin.  What this reaches is
// what the memory system gives that pattern (fewer, longer requests per wavefront and more concurrent
// streams than the plain copy above).
constexpr int kTilePieces = 17;
__global__ __launch_bounds__(256, 2) void k_tile_stream(f32x4c* __restrict__ w, int64_t ntiles, int tile_pieces, int S) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t nslabs = ntiles / S;
  const int64_t nw = (int64_t)gridDim.x * 4;
  for (int64_t slab = (int64_t)blockIdx.x * 4 + wave; slab < nslabs; slab += nw)
    for (int ts = 0; ts < S; ++ts) {
      f32x4c* t = w + (slab * S + ts) * tile_pieces;
      f32x4c v[kTilePieces];
#pragma unroll
      for (int i = 0; i < kTilePieces; ++i) {
        const int q = lane + i * 64;
        v[i] = __builtin_nontemporal_load(t + (q < tile_pieces ? q : tile_pieces - 1));
      }
#pragma unroll
      for (int i = 0; i < kTilePieces; ++i) asm volatile("" : "+v"(v[i]));   // every load before the first store
#pragma unroll
      for (int i = 0; i < kTilePieces; ++i) {
        const int q = lane + i * 64;
        if (q < tile_pieces) __builtin_nontemporal_store(v[i], t + q);
      }
    }
}

__global__ void k_zero_u32(uint32_t* p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

}  // namespace

void launch_copy16(hipStream_t s, void* dst, const void* src, int64_t n16) {
  if (n16 <= 0) return;
  const int64_t want = (n16 + 255) / 256;
  const unsigned grid = (unsigned)(want < 256 * 8 ? want : 256 * 8);
  k_copy16<<<dim3(grid), dim3(256), 0, s>>>(reinterpret_cast<f32x4c*>(dst), reinterpret_cast<const f32x4c*>(src), n16);
}

// `bytes` of `buf` as tiles of `tile_bytes` (a multiple of 16, at most 17 KB), slabs of `tiles_per_slab`;
// returns the bytes one launch reads (it writes as many): whole slabs only.
int64_t launch_tile_stream(hipStream_t s, void* buf, int64_t bytes, int tile_bytes, int tiles_per_slab, int cus) {
  const int tile_pieces = tile_bytes / 16;
  const int64_t ntiles = bytes / tile_bytes / tiles_per_slab * tiles_per_slab;
  if (ntiles <= 0) return 0;
  k_tile_stream<<<dim3((unsigned)(2 * cus)), dim3(256), 0, s>>>(reinterpret_cast<f32x4c*>(buf), ntiles, tile_pieces,
                                                            tiles_per_slab);
  return ntiles * (int64_t)tile_bytes;
}

void zero_u32(hipStream_t s, uint32_t* p, int64_t n) {
  if (n <= 0) return;
  k_zero_u32<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(p, n);
}

#define TGRAD_SEL_DISPATCH(KERN, GRID, BLOCK, ...)                                                    \
  do {                                                                                                \
    if (keys.random) KERN<kKeyRandom><<<dim3(GRID), dim3(BLOCK), 0, s>>>(__VA_ARGS__);                \
    else if (dtype == TGRAD_C64) KERN<TGRAD_C64><<<dim3(GRID), dim3(BLOCK), 0, s>>>(__VA_ARGS__);     \
    else KERN<TGRAD_CBF16><<<dim3(GRID), dim3(BLOCK), 0, s>>>(__VA_ARGS__);                           \
  } while (0)

void launch_select_hist(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                        uint32_t* hist) {
  int64_t npairs = I >> 1;
  int64_t want = (npairs + kSelThreads - 1) / kSelThreads;
  unsigned grid = (unsigned)(want < 1 ? 1 : want > 4096 ? 4096 : want);
  const KeySource src{g, keys.s0, keys.s1};
  TGRAD_SEL_DISPATCH(k_select_hist, grid, kSelThreads, src, I, hist);
}

void launch_select_pick(hipStream_t s, int pass, uint32_t k, SelectScalars* sc, const uint32_t* hist) {
  k_select_pick<<<dim3(1), dim3(1024), 0, s>>>(pass, k, sc, hist);
}

void launch_select_split(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                         const SelectScalars* sc, uint32_t* sure, uint32_t* cand) {
  const int64_t nseg = (I + kSegElems - 1) / kSegElems;
  unsigned grid = (unsigned)((nseg + kWavesPerBlock - 1) / kWavesPerBlock);
  const KeySource src{g, keys.s0, keys.s1};
  TGRAD_SEL_DISPATCH(k_select_split, grid, kSelThreads, src, I, sc, sure, cand, nseg);
}

void launch_select_hist_cand(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                             int pass, const SelectScalars* sc, const uint32_t* cand, uint32_t* hist) {
  const int64_t nwords = (I + 31) / 32;
  int64_t want = (nwords + kSelThreads - 1) / kSelThreads;
  unsigned grid = (unsigned)(want < 1 ? 1 : want > 2048 ? 2048 : want);
  const KeySource src{g, keys.s0, keys.s1};
  TGRAD_SEL_DISPATCH(k_select_hist_cand, grid, kSelThreads, src, pass, sc, cand, nwords, hist);
}

void launch_select_count(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                         const SelectScalars* sc, const uint32_t* sure, const uint32_t* cand,
                         uint32_t* chunk_gt, uint32_t* chunk_eq, int64_t nchunks) {
  const int64_t nwords = (I + 31) / 32;
  unsigned grid = (unsigned)((nchunks + kWavesPerBlock - 1) / kWavesPerBlock);
  const KeySource src{g, keys.s0, keys.s1};
  TGRAD_SEL_DISPATCH(k_select_count, grid, kSelThreads, src, sc, sure, cand, nwords, chunk_gt, chunk_eq, nchunks);
}

void launch_select_scan(hipStream_t s, uint32_t* chunk_gt, uint32_t* chunk_eq, int64_t nchunks) {
  k_select_scan<<<dim3(1), dim3(1024), 0, s>>>(chunk_gt, chunk_eq, nchunks);
}

void launch_select_emit(hipStream_t s, const void* g, int dtype, const SelectKeys& keys, int64_t I,
                        const SelectScalars* sc, const uint32_t* chunk_gt, const uint32_t* chunk_eq,
                        int64_t nchunks, uint32_t* sure, const uint32_t* cand, int32_t* omega) {
  const int64_t nwords = (I + 31) / 32;
  unsigned grid = (unsigned)((nchunks + kWavesPerBlock - 1) / kWavesPerBlock);
  const KeySource src{g, keys.s0, keys.s1};
  TGRAD_SEL_DISPATCH(k_select_emit, grid, kSelThreads, src, sc, chunk_gt, chunk_eq, nchunks, sure, cand, nwords,
                     omega);
}
#undef TGRAD_SEL_DISPATCH

void launch_mask_from_indices(hipStream_t s, const int32_t* omega, int64_t k, uint32_t* mask,
                              int64_t mask_words) {
  zero_u32(s, mask, mask_words);
  if (k > 0)
    k_mask_from_indices<<<dim3((unsigned)((k + 255) / 256)), dim3(256), 0, s>>>(omega, k, mask);
}

}  // namespace tgrad
