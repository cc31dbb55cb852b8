// Host side of the C ABI (include/tgrad.h): argument validation, the launch plan, carving of the
// caller's state / workspace buffers, and the sequencing of kernels on the caller's stream for
// the two branches of Algorithm 1 (refresh and step).
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "tgrad_internal.h"

namespace tgrad {
void zero_u32(hipStream_t s, uint32_t* p, int64_t n);
void launch_copy16(hipStream_t s, void* dst, const void* src, int64_t n16);
int64_t launch_tile_stream(hipStream_t s, void* buf, int64_t bytes, int tile_bytes, int tiles_per_slab, int cus);
void launch_eig_batch(hipStream_t s, int njobs, const double* const* gram, double* const* work_a,
                      double* const* work_v, const int* In, const int* r, float* const* U, int* const* status,
                      int max_sweeps);
void launch_identity_factor(hipStream_t s, float* U, int n);
}  // namespace tgrad

using namespace tgrad;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

const char* const kKernelNames[KID_COUNT] = {
    "select_hist", "select_pick", "select_split", "select_hist_cand", "select_count", "select_scan", "select_emit",
    "mask_from_indices",
    "tile_offsets", "gram", "gram_reduce", "eig_jacobi", "factor_pack",
    "gather", "project_first", "project", "adam_core", "backproject", "update", "sparse_update",
    "hooi_project", "core", "residual"};

struct Plan {
  int N = 0;
  int64_t I = 0;                 // elements of W / G
  int64_t C = 1;                 // elements of the core
  int64_t k = 0;
  int64_t shape[kMaxNdim];
  int rank[kMaxNdim];
  Stage proj[kMaxNdim];          // proj[s]: s-th projection stage; contracts mode N-1-s
  Stage back[kMaxNdim];          // back[s]: s-th reconstruction stage; expands mode s
  int64_t nchunks = 0;           // selection: runs of kSelChunkElems elements counted / emitted by one wavefront
  int64_t mask_words = 0;
  int tile_waves = 0;            // last-mode kernels: wavefronts per workgroup; 0 = generic kernels
  int64_t ntiles = 0;            // tiles of the tensor seen as (I / I_N rows, I_N)
  int64_t tile_elems = 0;
  bool fuse_next = false;        // the last-mode kernels also handle mode N-1 (see make_plan)
  bool fuse_core = false;        // last compression stage + AdamUpdate + first reconstruction stage in one kernel
  int fuse_core2 = 0;            // both leading modes, both ways, and AdamUpdate in one kernel (N = 4, see k_core2):
                                 // columns per workgroup (2 or 1), 0 = not used
  int core2_zgroup = 0;          // columns per unit of its result tensor (2 whenever the last rank is even)
  // byte offsets into state
  size_t st_omega, st_ms, st_vs, st_ml, st_vl, st_U[kMaxNdim], state_bytes;
  // byte offsets into workspace
  size_t ws_sel, ws_hist, ws_eig_status, ws_chunk_gt, ws_chunk_eq, ws_mask, ws_cand, ws_tile_start, ws_fpad, ws_ut, ws_core2, ws_partials, ws_gram[kMaxNdim],
      ws_eig_a[kMaxNdim], ws_eig_v[kMaxNdim], ws_gs, ws_core_g, ws_core_n, ws_buf[2], workspace_bytes;
  int gram_chunks[kMaxNdim];
  int order = 0;                   // TGRAD_ORDER_*
  size_t ws_tile_zero = 0;         // all-zero tile offsets: "no support" for the first-stage kernel
  size_t ws_resid = 0;             // low-rank-first order: the residual G - G~_L at refresh
  size_t ws_rbuf[2] = {0, 0};      // low-rank-first order: intermediates of the raw reconstruction chain
  int hooi_sweeps = 0;
  int hooi_gram_chunks[kMaxNdim];  // Gram of the chain result of mode n
};

// The stages of one HOOI projection chain: the residual compressed in every mode but `keep`
// (last mode first, like the step's own chain), then the extents of the result.
struct HooiChain {
  int nstages;
  Stage stage[kMaxNdim];
  int64_t out_elems[kMaxNdim];             // elements of each stage's output
  int64_t gram_A, gram_B;                  // the result viewed as (gram_A, I_keep, gram_B)
};

void hooi_chain(const Plan& p, int keep, HooiChain* ch) {
  int64_t cur[kMaxNdim];
  for (int m = 0; m < p.N; ++m) cur[m] = p.shape[m];
  ch->nstages = 0;
  for (int m = p.N - 1; m >= 0; --m) {
    if (m == keep) continue;
    Stage& st = ch->stage[ch->nstages];
    st.mode = m;
    st.A = 1;
    for (int j = 0; j < m; ++j) st.A *= cur[j];
    st.B = 1;
    for (int j = m + 1; j < p.N; ++j) st.B *= cur[j];
    st.K = (int)p.shape[m];
    st.M = p.rank[m];
    cur[m] = p.rank[m];
    ch->out_elems[ch->nstages] = st.A * st.M * st.B;
    ++ch->nstages;
  }
  ch->gram_A = 1;
  for (int j = 0; j < keep; ++j) ch->gram_A *= cur[j];
  ch->gram_B = 1;
  for (int j = keep + 1; j < p.N; ++j) ch->gram_B *= cur[j];
}

int validate(const tgrad_config* c) {
  if (!c) return TGRAD_ERR_INVALID_ARG;
  if (c->ndim < 2 || c->ndim > kMaxNdim) return TGRAD_ERR_INVALID_ARG;
  long double numel = 1;
  for (int n = 0; n < c->ndim; ++n) {
    if (c->shape[n] < 1) return TGRAD_ERR_INVALID_ARG;
    if (c->rank[n] < 1 || c->rank[n] > c->shape[n]) return TGRAD_ERR_INVALID_ARG;
    numel *= (long double)c->shape[n];
    if (numel >= 2147483648.0L) return TGRAD_ERR_UNSUPPORTED;
  }
  for (int n = 0; n < c->ndim; ++n)
    if (c->shape[n] > TGRAD_MAX_EXTENT && c->rank[n] != c->shape[n]) return TGRAD_ERR_UNSUPPORTED;
  if (c->k_sparse < 0 || (long double)c->k_sparse > numel) return TGRAD_ERR_INVALID_ARG;
  if (c->grad_dtype != TGRAD_C64 && c->grad_dtype != TGRAD_CBF16) return TGRAD_ERR_INVALID_ARG;
  if (c->weight_dtype != TGRAD_C64 && c->weight_dtype != TGRAD_CBF16) return TGRAD_ERR_INVALID_ARG;
  const float fl[] = {c->lr, c->beta1, c->beta2, c->eps, c->alpha, c->lambda, c->weight_decay};
  for (float f : fl)
    if (!std::isfinite(f)) return TGRAD_ERR_INVALID_ARG;
  if (c->beta1 < 0.f || c->beta1 >= 1.f || c->beta2 < 0.f || c->beta2 >= 1.f) return TGRAD_ERR_INVALID_ARG;
  if (c->eps < 0.f) return TGRAD_ERR_INVALID_ARG;
  if (c->refresh_every < 0) return TGRAD_ERR_INVALID_ARG;
  if (c->hooi_sweeps < 0 || c->hooi_sweeps > TGRAD_MAX_HOOI_SWEEPS) return TGRAD_ERR_INVALID_ARG;
  if (c->order != TGRAD_ORDER_US_LR && c->order != TGRAD_ORDER_LR_US && c->order != TGRAD_ORDER_SUM)
    return TGRAD_ERR_INVALID_ARG;
  if (c->eig_max_sweeps < 0 || c->eig_max_sweeps > TGRAD_MAX_EIG_SWEEPS) return TGRAD_ERR_INVALID_ARG;
  if (c->warm_restart != 0 && c->warm_restart != 1) return TGRAD_ERR_INVALID_ARG;
  if (c->warm_restart == 1 && c->hooi_sweeps < 1) return TGRAD_ERR_INVALID_ARG;
  if (c->select_rule != TGRAD_SELECT_TOPK_MAG && c->select_rule != TGRAD_SELECT_RANDOM)
    return TGRAD_ERR_INVALID_ARG;
  return TGRAD_OK;
}

void make_plan(const tgrad_config* c, Plan* p) {
  p->N = c->ndim;
  p->I = 1;
  p->C = 1;
  for (int n = 0; n < p->N; ++n) {
    p->shape[n] = c->shape[n];
    p->rank[n] = c->rank[n];
    p->I *= c->shape[n];
    p->C *= c->rank[n];
  }
  p->k = c->k_sparse;
  const int N = p->N;
  // projection: contract the last mode first (it is the contiguous one and the tensor shrinks
  // before the strided modes are touched); stage s handles mode n = N-1-s
  for (int s = 0; s < N; ++s) {
    const int n = N - 1 - s;
    Stage& st = p->proj[s];
    st.mode = n;
    st.A = 1;
    for (int m = 0; m < n; ++m) st.A *= p->shape[m];
    st.B = 1;
    for (int m = n + 1; m < N; ++m) st.B *= p->rank[m];
    st.K = (int)p->shape[n];
    st.M = p->rank[n];
  }
  // reconstruction: expand the first mode first, the last (contiguous) mode last, fused with W
  for (int s = 0; s < N; ++s) {
    Stage& st = p->back[s];
    st.mode = s;
    st.A = 1;
    for (int m = 0; m < s; ++m) st.A *= p->shape[m];
    st.B = 1;
    for (int m = s + 1; m < N; ++m) st.B *= p->rank[m];
    st.K = p->rank[s];
    st.M = (int)p->shape[s];
  }
  p->nchunks = (p->I + kSelChunkElems - 1) / kSelChunkElems;
  p->mask_words = (p->I + 31) / 32;
  {
    const int last = N - 1;
    p->tile_waves = choose_tile_waves((int)p->shape[last], p->rank[last], 4);
    if (c->weight_dtype == TGRAD_CBF16 && p->I < 4) p->tile_waves = 0;   // a bf16 tile needs one whole 16-byte piece
    const int64_t rows = p->I / p->shape[last];
    p->ntiles = (rows + 31) / 32;                 // last-mode kernels: flat tiles of 32 rows
    p->tile_elems = (int64_t)32 * p->shape[last];
    // Fusion of the mode-(N-1) stages into the last-mode kernels: needs whole 32-row tiles per slab,
    // one column tile of the last mode (r_N <= 16), r_(N-1) <= 32, and enough slabs to fill the chip.
    bool fuse = p->tile_waves == 4 && N >= 3;
    if (fuse) {
      const int64_t I2 = p->shape[last - 1];
      fuse = (I2 % 32 == 0) && I2 <= TGRAD_MAX_EXTENT && p->rank[last - 1] <= 32 && 2 * p->rank[last] <= 32 &&
             rows / I2 >= 512 && p->shape[last] <= fused_max_last_extent();
    }
    p->fuse_next = fuse;
    p->fuse_core = core_kernel_fits((int)p->shape[0], p->rank[0]);
    p->fuse_core2 = fuse && N == 4 ? core2_kernel_vec((int)p->shape[0], (int)p->shape[1], p->rank[0], p->rank[1],
                                                      p->rank[2], p->rank[3])
                                   : 0;
    p->core2_zgroup = p->fuse_core2 == 0 ? 0 : (p->rank[N - 1] % 2 == 0 ? 2 : 1);
  }

  size_t o = 0;
  auto take = [&o](size_t bytes) {
    size_t at = o;
    o = align_up(o + (bytes ? bytes : 1));
    return at;
  };
  p->st_omega = take((size_t)p->k * 4);
  p->st_ms = take((size_t)p->k * 8);
  p->st_vs = take((size_t)p->k * 4);
  p->st_ml = take((size_t)p->C * 8);
  p->st_vl = take((size_t)p->C * 4);
  for (int n = 0; n < N; ++n) p->st_U[n] = take((size_t)p->shape[n] * p->rank[n] * 8);
  p->state_bytes = o;

  o = 0;
  p->ws_sel = take(sizeof(SelectScalars));
  p->ws_hist = take(3 * kHistBins * 4);
  p->ws_eig_status = take(4 * kMaxNdim * sizeof(int));   // per mode: 1 if the last solve stopped at the sweep limit,
                                                         // Jacobi sweeps run, 1 if the tridiagonal path declined, spare
  p->ws_chunk_gt = take((size_t)p->nchunks * 4);
  p->ws_chunk_eq = take((size_t)p->nchunks * 4);
  p->ws_mask = take((size_t)p->mask_words * 4);
  p->ws_cand = take((size_t)p->mask_words * 4);
  p->ws_tile_start = take((size_t)(p->ntiles + 1) * 4);
  p->ws_fpad = take(p->fuse_next ? (size_t)p->shape[N - 2] * 32 * 8 : 0);
  p->ws_ut = take(p->fuse_next ? (size_t)p->shape[N - 2] * 32 * 8 : 0);
  p->ws_core2 = take(p->fuse_core2 ? core2_table_bytes((int)p->shape[1]) : 0);
  size_t partial_max = 0;
  for (int n = 0; n < N; ++n) {
    int64_t A = 1, B = 1;
    for (int m = 0; m < n; ++m) A *= p->shape[m];
    for (int m = n + 1; m < N; ++m) B *= p->shape[m];
    const bool compressed = p->rank[n] < p->shape[n];
    p->gram_chunks[n] = compressed ? gram_num_chunks(A, (int)p->shape[n], B) : 0;
    size_t bytes = (size_t)p->gram_chunks[n] * p->shape[n] * p->shape[n] * 16;
    if (bytes > partial_max) partial_max = bytes;
  }
  p->hooi_sweeps = c->hooi_sweeps;
  size_t hooi_buf[2] = {0, 0};
  for (int n = 0; n < N; ++n) {
    p->hooi_gram_chunks[n] = 0;
    if (p->hooi_sweeps == 0 || p->rank[n] == p->shape[n]) continue;
    HooiChain ch;
    hooi_chain(*p, n, &ch);
    for (int s = 0; s < ch.nstages; ++s) {
      const size_t b = (size_t)ch.out_elems[s] * 8;
      if (b > hooi_buf[s & 1]) hooi_buf[s & 1] = b;
    }
    p->hooi_gram_chunks[n] = gram_num_chunks(ch.gram_A, (int)p->shape[n], ch.gram_B);
    const size_t bytes = (size_t)p->hooi_gram_chunks[n] * p->shape[n] * p->shape[n] * 16;
    if (bytes > partial_max) partial_max = bytes;
  }
  p->ws_partials = take(partial_max);
  for (int n = 0; n < N; ++n) {
    const size_t mat = p->rank[n] < p->shape[n] ? (size_t)p->shape[n] * p->shape[n] * 16 : 0;
    p->ws_gram[n] = take(mat);
    p->ws_eig_a[n] = take(mat ? eig_work_bytes((int)p->shape[n]) : 0);
    p->ws_eig_v[n] = take(mat);
  }
  p->ws_gs = take((size_t)p->k * 8);
  p->ws_core_g = take((size_t)p->C * 8);
  p->ws_core_n = take((size_t)p->C * 8);
  size_t buf[2] = {hooi_buf[0], hooi_buf[1]};
  for (int s = 0; s + 1 < N; ++s) {
    size_t bp = (size_t)(p->proj[s].A * p->proj[s].M * p->proj[s].B) * 8;
    size_t bb = (size_t)(p->back[s].A * p->back[s].M * p->back[s].B) * 8;
    if (bp > buf[s & 1]) buf[s & 1] = bp;
    if (bb > buf[s & 1]) buf[s & 1] = bb;
  }
  p->ws_buf[0] = take(buf[0]);
  p->ws_buf[1] = take(buf[1]);
  p->order = c->order;
  p->ws_tile_zero = take(p->order != TGRAD_ORDER_US_LR ? (size_t)(p->ntiles + 1) * 4 : 0);
  {
    // unfused chains (every stage through memory) for the residual of the low-rank part
    size_t rb[2] = {0, 0};
    if (p->order == TGRAD_ORDER_LR_US) {
      for (int s = 0; s + 1 < N; ++s) {
        size_t bp = (size_t)(p->proj[s].A * p->proj[s].M * p->proj[s].B) * 8;
        size_t bb = (size_t)(p->back[s].A * p->back[s].M * p->back[s].B) * 8;
        if (bp > rb[s & 1]) rb[s & 1] = bp;
        if (bb > rb[s & 1]) rb[s & 1] = bb;
      }
    }
    p->ws_rbuf[0] = take(rb[0]);
    p->ws_rbuf[1] = take(rb[1]);
    p->ws_resid = take(p->order == TGRAD_ORDER_LR_US ? (size_t)p->I * 8 : 0);
  }
  p->workspace_bytes = o;
}

struct EventPair {
  hipEvent_t a, b;
  int kid;
};

}  // namespace

struct tgrad_ctx {
  tgrad_config cfg;
  Plan plan;
  char* state;
  char* ws;
  hipStream_t stream;
  int64_t t;
  bool have_indices;
  bool have_factor[kMaxNdim];
  bool have_hist;                 // the leading-digit histogram of the last refresh's gradient is in the workspace
  int launch_status;              // first failed kernel launch of the current call (TGRAD_OK = none)
  bool profiling;
  std::vector<EventPair> events;
  double total_ms[KID_COUNT];
  int64_t launches[KID_COUNT];

  template <typename T>
  T* st(size_t off) { return reinterpret_cast<T*>(state + off); }
  template <typename T>
  T* w(size_t off) { return reinterpret_cast<T*>(ws + off); }
  bool ready() const {
    if (!have_indices) return false;
    for (int n = 0; n < plan.N; ++n)
      if (!have_factor[n]) return false;
    return true;
  }
};

namespace {

// Brackets one kernel launch with events when profiling is on.
struct Scope {
  tgrad_ctx* c;
  int kid;
  hipEvent_t a = nullptr, b = nullptr;
  Scope(tgrad_ctx* ctx, int k) : c(ctx), kid(k) {
    if (c->profiling && c->events.size() < 200000) {
      if (hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess) {
        (void)hipEventRecord(a, c->stream);
      } else {
        a = b = nullptr;
      }
    }
  }
  ~Scope() {
    // every launch is checked where it happens, so a failure is charged to the call (and kernel)
    // that caused it
    if (hipGetLastError() != hipSuccess && c->launch_status == TGRAD_OK) c->launch_status = TGRAD_ERR_HIP;
    if (a && b) {
      (void)hipEventRecord(b, c->stream);
      c->events.push_back({a, b, kid});
    }
  }
};

int drain_events(tgrad_ctx* c) {
  if (hipStreamSynchronize(c->stream) != hipSuccess) return TGRAD_ERR_HIP;
  for (auto& e : c->events) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, e.a, e.b) == hipSuccess) {
      c->total_ms[e.kid] += ms;
      c->launches[e.kid] += 1;
    }
    (void)hipEventDestroy(e.a);
    (void)hipEventDestroy(e.b);
  }
  c->events.clear();
  return TGRAD_OK;
}

int check_launch() { return hipGetLastError() == hipSuccess ? TGRAD_OK : TGRAD_ERR_HIP; }

// Status of the launches of the call that is ending: the first failure a Scope saw, else whatever the
// runtime still reports (launches outside a Scope); the per-call record is cleared.
int finish_call(tgrad_ctx* c) {
  const int tail = check_launch();
  const int rc = c->launch_status != TGRAD_OK ? c->launch_status : tail;
  c->launch_status = TGRAD_OK;
  return rc;
}

// An error that was pending in the runtime BEFORE this library launched anything belongs to the
// caller: it is reported (not cleared, so the caller still finds it) and nothing is launched.
bool error_pending_on_entry() { return hipPeekAtLastError() != hipSuccess; }

// Kernel-ready copies of U^(N-1) for the fused kernels, and of U^(1), U^(2) for the two-mode core kernel;
// rebuilt whenever a factor changes (refresh, HOOI sweep, tgrad_set_state), never on the step path.
void pack_fused_factor(tgrad_ctx* c) {
  Plan& p = c->plan;
  if (!p.fuse_next) return;
  Scope sc_(c, KID_FACTOR_PACK);
  launch_pack_fused_factor(c->stream, c->st<float2>(p.st_U[p.N - 2]), (int)p.shape[p.N - 2], p.rank[p.N - 2],
                           c->w<float2>(p.ws_fpad), c->w<float2>(p.ws_ut));
  if (p.fuse_core2)
    launch_pack_core2(c->stream, c->st<float2>(p.st_U[0]), p.rank[0], p.rank[0], c->st<float2>(p.st_U[1]), p.rank[1],
                      p.rank[1], (int)p.shape[1], c->w<float2>(p.ws_core2));
}

// Omega <- SparseIndices(x, rho, top-k | rand-k), plus the support bitmask and the tile offsets.
void select_support(tgrad_ctx* c, const void* x, int dt) {
  Plan& p = c->plan;
  hipStream_t s = c->stream;
  SelectScalars* sc = c->w<SelectScalars>(p.ws_sel);
  uint32_t* hist = c->w<uint32_t>(p.ws_hist);
  uint32_t* chunk_gt = c->w<uint32_t>(p.ws_chunk_gt);
  uint32_t* chunk_eq = c->w<uint32_t>(p.ws_chunk_eq);
  uint32_t* mask = c->w<uint32_t>(p.ws_mask);          // "sure" bits first, the support bitmask in the end
  uint32_t* cand = c->w<uint32_t>(p.ws_cand);
  int32_t* omega = c->st<int32_t>(p.st_omega);
  SelectKeys keys{false, 0u, 0u};
  if (c->cfg.select_rule == TGRAD_SELECT_RANDOM) {
    const uint64_t seed = c->cfg.select_seed;
    const uint32_t t32 = (uint32_t)((uint64_t)c->t & 0xFFFFFFFFull);
    keys.random = true;
    keys.s0 = (uint32_t)(seed & 0xFFFFFFFFull) ^ (t32 * 0x9E3779B9u);
    keys.s1 = (uint32_t)(seed >> 32) + t32 + 0x7F4A7C15u;
  }
  if (p.k > 0) {
    zero_u32(s, hist, 3 * kHistBins);
    // two streaming passes over x: leading-digit histogram, then the two bitmasks
    { Scope sc_(c, KID_SEL_HIST); launch_select_hist(s, x, dt, keys, p.I, hist); }
    { Scope sc_(c, KID_SEL_PICK); launch_select_pick(s, 0, (uint32_t)p.k, sc, hist); }
    { Scope sc_(c, KID_SEL_SPLIT); launch_select_split(s, x, dt, keys, p.I, sc, mask, cand); }
    // the remaining digits are decided among the candidates only
    for (int pass = 1; pass < 3; ++pass) {
      { Scope sc_(c, KID_SEL_HIST_CAND); launch_select_hist_cand(s, x, dt, keys, p.I, pass, sc, cand, hist + pass * kHistBins); }
      { Scope sc_(c, KID_SEL_PICK); launch_select_pick(s, pass, (uint32_t)p.k, sc, hist + pass * kHistBins); }
    }
    { Scope sc_(c, KID_SEL_COUNT); launch_select_count(s, x, dt, keys, p.I, sc, mask, cand, chunk_gt, chunk_eq, p.nchunks); }
    { Scope sc_(c, KID_SEL_SCAN); launch_select_scan(s, chunk_gt, chunk_eq, p.nchunks); }
    { Scope sc_(c, KID_SEL_EMIT); launch_select_emit(s, x, dt, keys, p.I, sc, chunk_gt, chunk_eq, p.nchunks, mask, cand, omega); }
  }
  c->have_hist = p.k > 0 && !keys.random;
  {
    Scope sc_(c, KID_TILE_OFFSETS);
    launch_tile_offsets(s, omega, p.k, p.tile_elems, p.ntiles, c->w<uint32_t>(p.ws_tile_start));
  }
  c->have_indices = true;
}

// First stage of a compression chain that reads G itself.  `tile_start` / `use_mask` say which
// support is removed on the way in: the real one, or none (all-zero offsets, null mask).
void first_stage(tgrad_ctx* c, const void* g, const Stage& sg, const uint32_t* tile_start, const uint32_t* use_mask,
                 float2* dst) {
  Plan& p = c->plan;
  const float2* Um = c->st<float2>(p.st_U[sg.mode]);
  if (sg.mode == p.N - 1 && p.tile_waves > 0)
    launch_lproj(c->stream, g, c->cfg.grad_dtype, c->st<int32_t>(p.st_omega), tile_start, c->w<float2>(p.ws_gs), Um,
                 sg.M, sg, p.tile_waves, dst, 0, 0, nullptr);
  else
    launch_contract(c->stream, g, c->cfg.grad_dtype, use_mask, Um, sg.K, sg.M, true, sg, dst);
}

// {U^(n)} <- TuckerFactors(G with the given support removed, r): HOSVD (or the factors in place,
// warm restart), then the HOOI sweeps.
void compute_factors(tgrad_ctx* c, const void* g, const uint32_t* tile_start, const uint32_t* use_mask) {
  Plan& p = c->plan;
  hipStream_t s = c->stream;
  const int dt = c->cfg.grad_dtype;
  // Warm restart: the sweeps below start from the factors in place instead of from HOSVD.
  bool warm = c->cfg.warm_restart == 1 && p.hooi_sweeps > 0;
  for (int n = 0; n < p.N; ++n) warm = warm && c->have_factor[n];
  const double* grams[kMaxNdim];
  double* wa[kMaxNdim];
  double* wv[kMaxNdim];
  int In[kMaxNdim], rr[kMaxNdim];
  float* Us[kMaxNdim];
  int* stat[kMaxNdim];
  int njobs = 0;
  for (int n = 0; n < p.N; ++n) {
    float* U = c->st<float>(p.st_U[n]);
    if (p.rank[n] == p.shape[n]) {
      Scope sc_(c, KID_FACTOR_PACK);
      launch_identity_factor(s, U, (int)p.shape[n]);
    } else if (!warm) {
      int64_t A = 1, B = 1;
      for (int m = 0; m < n; ++m) A *= p.shape[m];
      for (int m = n + 1; m < p.N; ++m) B *= p.shape[m];
      double* partials = c->w<double>(p.ws_partials);
      double* gram = c->w<double>(p.ws_gram[n]);
      { Scope sc_(c, KID_GRAM); launch_gram(s, g, dt, use_mask, A, (int)p.shape[n], B, p.gram_chunks[n], partials); }
      { Scope sc_(c, KID_GRAM_REDUCE); launch_gram_reduce(s, partials, p.gram_chunks[n], (int)p.shape[n], gram); }
      grams[njobs] = gram;
      wa[njobs] = c->w<double>(p.ws_eig_a[n]);
      wv[njobs] = c->w<double>(p.ws_eig_v[n]);
      In[njobs] = (int)p.shape[n];
      rr[njobs] = p.rank[n];
      Us[njobs] = U;
      stat[njobs] = c->w<int>(p.ws_eig_status) + 4 * n;
      ++njobs;
    }
    c->have_factor[n] = true;
  }
  if (njobs > 0) {
    Scope sc_(c, KID_EIG);
    launch_eig_batch(s, njobs, grams, wa, wv, In, rr, Us, stat, c->cfg.eig_max_sweeps);
  }

  // --- HOOI sweeps: mode n re-solved on the tensor compressed in every other mode ---
  float2* buf[2] = {c->w<float2>(p.ws_buf[0]), c->w<float2>(p.ws_buf[1])};
  for (int sweep = 0; sweep < p.hooi_sweeps; ++sweep) {
    for (int n = 0; n < p.N; ++n) {
      if (p.rank[n] == p.shape[n]) continue;
      HooiChain ch;
      hooi_chain(p, n, &ch);
      const float2* src = nullptr;
      for (int st = 0; st < ch.nstages; ++st) {
        const Stage& sg = ch.stage[st];
        float2* dst = buf[st & 1];
        Scope sc_(c, KID_HOOI_PROJECT);
        if (st == 0)
          first_stage(c, g, sg, tile_start, use_mask, dst);
        else
          launch_mid(s, src, c->st<float2>(p.st_U[sg.mode]), sg.M, true, sg, dst);
        src = dst;
      }
      double* partials = c->w<double>(p.ws_partials);
      double* gram = c->w<double>(p.ws_gram[n]);
      { Scope sc_(c, KID_GRAM); launch_gram(s, src, TGRAD_C64, nullptr, ch.gram_A, (int)p.shape[n], ch.gram_B, p.hooi_gram_chunks[n], partials); }
      { Scope sc_(c, KID_GRAM_REDUCE); launch_gram_reduce(s, partials, p.hooi_gram_chunks[n], (int)p.shape[n], gram); }
      const double* g1[1] = {gram};
      double* a1[1] = {c->w<double>(p.ws_eig_a[n])};
      double* v1[1] = {c->w<double>(p.ws_eig_v[n])};
      int i1[1] = {(int)p.shape[n]}, r1[1] = {p.rank[n]};
      float* u1[1] = {c->st<float>(p.st_U[n])};
      int* s1[1] = {c->w<int>(p.ws_eig_status) + 4 * n};
      Scope sc_(c, KID_EIG);
      launch_eig_batch(s, 1, g1, a1, v1, i1, r1, u1, s1, c->cfg.eig_max_sweeps);
    }
  }
  pack_fused_factor(c);
}

// z = (G~_L before its last expansion), (A, r_N): the core `core` expanded in modes 1 .. N-1 through the
// buffers of the raw chain.  Returns where it lies.
const float2* raw_expand(tgrad_ctx* c, const float2* core) {
  Plan& p = c->plan;
  float2* rb[2] = {c->w<float2>(p.ws_rbuf[0]), c->w<float2>(p.ws_rbuf[1])};
  const float2* src = core;
  for (int st = 0; st + 1 < p.N; ++st) {
    const Stage& sg = p.back[st];
    float2* dst = rb[st & 1];
    Scope sc_(c, KID_RESIDUAL);
    launch_mid(c->stream, src, c->st<float2>(p.st_U[sg.mode]), p.rank[sg.mode], false, sg, dst);
    src = dst;
  }
  return src;
}

int do_refresh(tgrad_ctx* c, const void* g) {
  Plan& p = c->plan;
  hipStream_t s = c->stream;
  const int dt = c->cfg.grad_dtype;
  const uint32_t* real_ts = c->w<uint32_t>(p.ws_tile_start);
  if (p.order == TGRAD_ORDER_US_LR) {
    // Algorithm 1: support from G, factors from G with the support removed
    select_support(c, g, dt);
    compute_factors(c, g, real_ts, p.k > 0 ? c->w<uint32_t>(p.ws_mask) : nullptr);
    return finish_call(c);
  }
  const uint32_t* zero_ts = c->w<uint32_t>(p.ws_tile_zero);
  if (p.order == TGRAD_ORDER_SUM) {
    // both components see the full gradient
    select_support(c, g, dt);
    compute_factors(c, g, zero_ts, nullptr);
    return finish_call(c);
  }
  // low rank first: factors of the full gradient, then the support from R = G - G~_L
  compute_factors(c, g, zero_ts, nullptr);
  float2* rb[2] = {c->w<float2>(p.ws_rbuf[0]), c->w<float2>(p.ws_rbuf[1])};
  float2* core = c->w<float2>(p.ws_core_g);
  const float2* src = nullptr;
  for (int st = 0; st < p.N; ++st) {                           // unfused compression chain, nothing removed
    const Stage& sg = p.proj[st];
    float2* dst = (st == p.N - 1) ? core : rb[st & 1];
    Scope sc_(c, KID_RESIDUAL);
    if (st == 0)
      first_stage(c, g, sg, zero_ts, nullptr, dst);
    else
      launch_mid(s, src, c->st<float2>(p.st_U[sg.mode]), p.rank[sg.mode], true, sg, dst);
    src = dst;
  }
  const float2* z = raw_expand(c, core);
  {
    const Stage& sg = p.back[p.N - 1];
    Scope sc_(c, KID_RESIDUAL);
    launch_residual(s, g, dt, z, c->st<float2>(p.st_U[p.N - 1]), p.rank[p.N - 1], sg.A, sg.M, c->w<float2>(p.ws_resid));
  }
  select_support(c, c->w<float2>(p.ws_resid), TGRAD_C64);
  return finish_call(c);
}

int do_step(tgrad_ctx* c, void* weight, const void* g) {
  Plan& p = c->plan;
  const tgrad_config& cf = c->cfg;
  hipStream_t s = c->stream;
  const int N = p.N;
  const int32_t* omega = c->st<int32_t>(p.st_omega);
  const uint32_t* mask = p.k > 0 ? c->w<uint32_t>(p.ws_mask) : nullptr;
  float2* gs = c->w<float2>(p.ws_gs);
  float2* core_g = c->w<float2>(p.ws_core_g);
  float2* core_n = c->w<float2>(p.ws_core_n);
  float2* buf[2] = {c->w<float2>(p.ws_buf[0]), c->w<float2>(p.ws_buf[1])};

  const uint32_t* tile_start = c->w<uint32_t>(p.ws_tile_start);
  const bool mfma_last = p.tile_waves > 0;
  // What the compression chain removes on the way in: the support (Algorithm 1), or nothing (the
  // low-rank part sees the full gradient in the two other composition orders).
  const bool remove_support = p.order == TGRAD_ORDER_US_LR;
  const uint32_t* in_ts = remove_support ? tile_start : c->w<uint32_t>(p.ws_tile_zero);
  const uint32_t* in_mask = remove_support ? mask : nullptr;

  // g_S <- Sparse(G, Omega);  g_L <- (G - g_S) x_N UN^H ... x_1 U1^H
  // (the matrix-core first stage gathers the values it removes; otherwise a gather kernel does)
  if (!mfma_last || !remove_support) { Scope sc_(c, KID_GATHER); launch_gather(s, g, cf.grad_dtype, omega, p.k, gs); }
  const float2* src = nullptr;
  for (int st = 0; st < N; ++st) {
    const Stage& sg = p.proj[st];
    float2* dst = (st == N - 1) ? core_g : buf[st & 1];
    const float2* U = c->st<float2>(p.st_U[sg.mode]);
    if (st == 0 && mfma_last && p.fuse_next) {                 // stages 0 and 1 in one kernel
      float2* dst1 = (N == 2) ? core_g : buf[1];
      Scope sc_(c, KID_PROJECT_FIRST);
      launch_lproj(s, g, cf.grad_dtype, omega, in_ts, gs, U, p.rank[sg.mode], sg, p.tile_waves, dst1,
                   (int)p.shape[N - 2], p.rank[N - 2], c->w<float2>(p.ws_fpad));
      src = dst1;
      st = 1;
      continue;
    }
    if (st == N - 2 && p.fuse_core2) break;                    // modes 2 and 1 are contracted inside k_core2 below
    if (st == N - 1 && p.fuse_core) break;                     // mode 1 is contracted inside k_core below
    Scope sc_(c, st == 0 ? KID_PROJECT_FIRST : KID_PROJECT);
    if (st == 0) {
      if (mfma_last)
        launch_lproj(s, g, cf.grad_dtype, omega, in_ts, gs, U, p.rank[sg.mode], sg, p.tile_waves, dst, 0, 0,
                     nullptr);
      else
        launch_contract(s, g, cf.grad_dtype, in_mask, U, (int)p.shape[sg.mode], p.rank[sg.mode], true, sg, dst);
    } else {
      launch_mid(s, src, U, p.rank[sg.mode], true, sg, dst);
    }
    src = dst;
  }

  // AdamUpdate on the core; tau = t + 1
  const double tau = (double)(c->t + 1);
  const float inv_c1 = (float)(1.0 / (1.0 - std::pow((double)cf.beta1, tau)));
  const float inv_c2 = (float)(1.0 / (1.0 - std::pow((double)cf.beta2, tau)));
  const float2* zsrc = core_n;
  int first_back = 0;
  if (p.fuse_core2) {
    // the last two compression stages, AdamUpdate on the core and the first two reconstruction stages
    Scope sc_(c, KID_CORE);
    launch_core2(s, p.fuse_core2, p.core2_zgroup, src, c->w<float2>(p.ws_core2), (int)p.shape[1], p.rank[0], p.rank[1],
                 (int64_t)p.rank[2] * p.rank[3], c->st<float2>(p.st_ml), c->st<float>(p.st_vl), core_g, cf.beta1,
                 cf.beta2, inv_c1, inv_c2, cf.eps, buf[0]);
    zsrc = buf[0];
    first_back = 2;
  } else if (p.fuse_core) {
    // last compression stage, AdamUpdate on the core and first reconstruction stage (all mode 1)
    const Stage& sg = p.proj[N - 1];
    Scope sc_(c, KID_CORE);
    launch_core(s, src, c->st<float2>(p.st_U[0]), p.rank[0], sg.K, sg.M, sg.B, c->st<float2>(p.st_ml),
                c->st<float>(p.st_vl), core_g, cf.beta1, cf.beta2, inv_c1, inv_c2, cf.eps, buf[0]);
    zsrc = buf[0];
    first_back = 1;
  } else {
    Scope sc_(c, KID_ADAM_CORE);
    launch_adam_core(s, core_g, c->st<float2>(p.st_ml), c->st<float>(p.st_vl), core_n, p.C, cf.beta1,
                     cf.beta2, inv_c1, inv_c2, cf.eps);
  }

  // low rank first: the sparse part works on the residual of the low-rank approximation of THIS
  // gradient: g_S <- g_S - (g_L x_1 U1 ... x_N UN)[Omega]
  if (p.order == TGRAD_ORDER_LR_US && p.k > 0) {
    const float2* z = raw_expand(c, core_g);
    Scope sc_(c, KID_RESIDUAL);
    launch_residual_gather(s, gs, omega, p.k, z, c->st<float2>(p.st_U[N - 1]), p.rank[N - 1], (int)p.shape[N - 1]);
  }

  // D <- alpha (N_L x_1 U1 ... x_N UN); the last stage is fused with AdamUpdate on the sparse values,
  // D[Omega] += lambda N_S and W <- W (1 - lr wd) - lr D
  const int nmid = (mfma_last && p.fuse_next) ? N - 2 : N - 1;   // reconstruction stages run by k_mid
  for (int st = first_back; st < nmid; ++st) {
    const Stage& sg = p.back[st];
    float2* dst = buf[st & 1];
    const float2* U = c->st<float2>(p.st_U[sg.mode]);
    Scope sc_(c, KID_BACKPROJECT);
    launch_mid(s, zsrc, U, p.rank[sg.mode], false, sg, dst);
    zsrc = dst;
  }
  {
    const Stage& sg = p.back[N - 1];
    const float2* U = c->st<float2>(p.st_U[sg.mode]);
    const float decay = 1.f - cf.lr * cf.weight_decay;
    if (mfma_last && p.fuse_next) {
      Scope sc_(c, KID_UPDATE);
      launch_lupdate_fused(s, zsrc, c->w<float2>(p.ws_ut), (int)p.shape[N - 2], p.rank[N - 2], U, sg,
                           weight, cf.weight_dtype, decay, -cf.lr * cf.alpha, omega, tile_start, p.k, gs,
                           c->st<float2>(p.st_ms), c->st<float>(p.st_vs), cf.beta1, cf.beta2, inv_c1, inv_c2,
                           cf.eps, -cf.lr * cf.lambda, p.core2_zgroup);
    } else if (mfma_last) {
      Scope sc_(c, KID_UPDATE);
      launch_lupdate(s, zsrc, U, sg, p.tile_waves, weight, cf.weight_dtype, decay, -cf.lr * cf.alpha,
                     omega, tile_start, gs, c->st<float2>(p.st_ms), c->st<float>(p.st_vs), cf.beta1, cf.beta2,
                     inv_c1, inv_c2, cf.eps, -cf.lr * cf.lambda);
    } else {
      {
        Scope sc_(c, KID_SPARSE_UPDATE);
        launch_sparse_adam(s, gs, p.k, c->st<float2>(p.st_ms), c->st<float>(p.st_vs), cf.beta1, cf.beta2, inv_c1,
                           inv_c2, cf.eps, -cf.lr * cf.lambda);
      }
      Scope sc_(c, KID_UPDATE);
      launch_update(s, zsrc, U, (int)p.shape[sg.mode], p.rank[sg.mode], sg, weight, cf.weight_dtype, decay,
                    -cf.lr * cf.alpha, mask, omega, p.k, gs);
    }
  }
  c->t += 1;
  return finish_call(c);
}

struct Item {
  char* dev;        // device address
  size_t bytes;     // bytes on the device == bytes on the host (except INDICES)
  bool writable;
  bool needs_indices, needs_factor;
  int mode;
};

int locate(tgrad_ctx* c, int what, Item* it) {
  Plan& p = c->plan;
  it->writable = true;
  it->needs_indices = it->needs_factor = false;
  it->mode = -1;
  switch (what) {
    case TGRAD_STATE_CORE_M: it->dev = c->state + p.st_ml; it->bytes = (size_t)p.C * 8; return TGRAD_OK;
    case TGRAD_STATE_CORE_V: it->dev = c->state + p.st_vl; it->bytes = (size_t)p.C * 4; return TGRAD_OK;
    case TGRAD_STATE_SPARSE_M: it->dev = c->state + p.st_ms; it->bytes = (size_t)p.k * 8; return TGRAD_OK;
    case TGRAD_STATE_SPARSE_V: it->dev = c->state + p.st_vs; it->bytes = (size_t)p.k * 4; return TGRAD_OK;
    case TGRAD_STATE_SPARSE_G: it->dev = c->ws + p.ws_gs; it->bytes = (size_t)p.k * 8; it->writable = false; return TGRAD_OK;
    case TGRAD_STATE_CORE_G: it->dev = c->ws + p.ws_core_g; it->bytes = (size_t)p.C * 8; it->writable = false; return TGRAD_OK;
    default: break;
  }
  if (what >= TGRAD_STATE_FACTOR0 && what < TGRAD_STATE_FACTOR0 + p.N) {
    const int n = what - TGRAD_STATE_FACTOR0;
    it->dev = c->state + p.st_U[n];
    it->bytes = (size_t)p.shape[n] * p.rank[n] * 8;
    it->needs_factor = true;
    it->mode = n;
    return TGRAD_OK;
  }
  if (what >= TGRAD_STATE_EIG_INFO0 && what < TGRAD_STATE_EIG_INFO0 + p.N) {
    const int n = what - TGRAD_STATE_EIG_INFO0;
    if (p.rank[n] == p.shape[n]) return TGRAD_ERR_INVALID_ARG;     // identity factor: nothing is solved
    it->dev = c->ws + p.ws_eig_status + (size_t)4 * n * sizeof(int);
    it->bytes = 3 * sizeof(int);
    it->writable = false;
    it->needs_factor = true;
    it->mode = n;
    return TGRAD_OK;
  }
  if (what >= TGRAD_STATE_GRAM0 && what < TGRAD_STATE_GRAM0 + p.N) {
    const int n = what - TGRAD_STATE_GRAM0;
    if (p.rank[n] == p.shape[n]) return TGRAD_ERR_INVALID_ARG;     // no Gram is formed for an uncompressed mode
    it->dev = c->ws + p.ws_gram[n];
    it->bytes = (size_t)p.shape[n] * p.shape[n] * 16;
    it->writable = false;
    it->needs_factor = true;
    it->mode = n;
    return TGRAD_OK;
  }
  return TGRAD_ERR_INVALID_ARG;
}

// ---- workspace of tgrad_step_static ------------------------------------------------------------
// One fixed array per GPU (every GPU the code object is loaded on holds its own copy until the
// process ends).  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address is looked up once per device and every kernel receives that address.
__device__ __align__(256) unsigned char g_static_workspace[TGRAD_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void* g_static_ptr[kMaxDevices];          // device address of g_static_workspace, per device; null = not looked up yet

int static_workspace(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TGRAD_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_workspace)) != hipSuccess || !ptr) return TGRAD_ERR_HIP;
    g_static_ptr[dev] = ptr;
  }
  *out = g_static_ptr[dev];
  return TGRAD_OK;
}

}  // namespace

extern "C" {

int tgrad_query_sizes(const tgrad_config* cfg, size_t* state_bytes, size_t* workspace_bytes) {
  if (!state_bytes || !workspace_bytes) return TGRAD_ERR_INVALID_ARG;
  int rc = validate(cfg);
  if (rc != TGRAD_OK) return rc;
  Plan p;
  make_plan(cfg, &p);
  *state_bytes = p.state_bytes;
  *workspace_bytes = p.workspace_bytes;
  return TGRAD_OK;
}

int tgrad_init(tgrad_ctx** out, const tgrad_config* cfg, void* state_dev, void* workspace_dev,
               void* hip_stream) {
  if (!out) return TGRAD_ERR_INVALID_ARG;
  *out = nullptr;
  int rc = validate(cfg);
  if (rc != TGRAD_OK) return rc;
  if (!state_dev || !workspace_dev) return TGRAD_ERR_INVALID_ARG;
  if (((uintptr_t)state_dev % kAlign) || ((uintptr_t)workspace_dev % kAlign)) return TGRAD_ERR_INVALID_ARG;
  tgrad_ctx* c = new (std::nothrow) tgrad_ctx();
  if (!c) return TGRAD_ERR_INVALID_ARG;
  c->cfg = *cfg;
  make_plan(cfg, &c->plan);
  c->state = static_cast<char*>(state_dev);
  c->ws = static_cast<char*>(workspace_dev);
  c->stream = static_cast<hipStream_t>(hip_stream);
  c->t = 0;
  c->have_indices = false;
  for (int n = 0; n < kMaxNdim; ++n) c->have_factor[n] = false;
  c->have_hist = false;
  c->launch_status = TGRAD_OK;
  c->profiling = false;
  for (int i = 0; i < KID_COUNT; ++i) {
    c->total_ms[i] = 0.;
    c->launches[i] = 0;
  }
  // no solve has hit its sweep limit yet (a factor injected with tgrad_set_state never does)
  zero_u32(c->stream, c->w<uint32_t>(c->plan.ws_eig_status), 4 * kMaxNdim);
  // moments <- 0 (and everything else in the state block), with a fill kernel
  zero_u32(c->stream, reinterpret_cast<uint32_t*>(c->state), (int64_t)(c->plan.state_bytes / 4));
  if (c->plan.order != TGRAD_ORDER_US_LR)
    zero_u32(c->stream, c->w<uint32_t>(c->plan.ws_tile_zero), c->plan.ntiles + 1);
  if (check_launch() != TGRAD_OK) {
    delete c;
    return TGRAD_ERR_HIP;
  }
  *out = c;
  return TGRAD_OK;
}

int tgrad_refresh_factors(tgrad_ctx* ctx, const void* grad_dev) {
  if (!ctx || !grad_dev) return TGRAD_ERR_INVALID_ARG;
  if ((uintptr_t)grad_dev % 16) return TGRAD_ERR_INVALID_ARG;
  if (error_pending_on_entry()) return TGRAD_ERR_HIP;
  return do_refresh(ctx, grad_dev);
}

int tgrad_step(tgrad_ctx* ctx, void* weight_dev, const void* grad_dev) {
  if (!ctx || !weight_dev || !grad_dev) return TGRAD_ERR_INVALID_ARG;
  if (((uintptr_t)grad_dev % 16) || ((uintptr_t)weight_dev % 16) || weight_dev == grad_dev)
    return TGRAD_ERR_INVALID_ARG;
  if (error_pending_on_entry()) return TGRAD_ERR_HIP;
  if (ctx->cfg.refresh_every > 0 && ctx->t % ctx->cfg.refresh_every == 0) {
    int rc = do_refresh(ctx, grad_dev);
    if (rc != TGRAD_OK) return rc;
  }
  if (!ctx->ready()) return TGRAD_ERR_NOT_READY;
  return do_step(ctx, weight_dev, grad_dev);
}

int tgrad_step_static(const tgrad_config* cfg, void* state_dev, int64_t t, void* weight_dev,
                      const void* grad_dev, void* hip_stream) {
  int rc = validate(cfg);
  if (rc != TGRAD_OK) return rc;
  if (!state_dev || !weight_dev || !grad_dev || t < 0) return TGRAD_ERR_INVALID_ARG;
  if (((uintptr_t)state_dev % kAlign) || ((uintptr_t)grad_dev % 16) || ((uintptr_t)weight_dev % 16) ||
      weight_dev == grad_dev)
    return TGRAD_ERR_INVALID_ARG;
  if (cfg->refresh_every < 1) return TGRAD_ERR_INVALID_ARG;      // nobody else could refresh this state
  tgrad_ctx c;                                                    // on the stack: nothing is allocated
  c.cfg = *cfg;
  make_plan(cfg, &c.plan);
  if (c.plan.workspace_bytes > (size_t)TGRAD_STATIC_WORKSPACE_BYTES) return TGRAD_ERR_UNSUPPORTED;
  void* ws = nullptr;
  rc = static_workspace(&ws);
  if (rc != TGRAD_OK) return rc;
  c.state = static_cast<char*>(state_dev);
  c.ws = static_cast<char*>(ws);
  c.stream = static_cast<hipStream_t>(hip_stream);
  c.t = t;
  c.have_indices = true;                                          // the caller's contract for t % T != 0
  for (int n = 0; n < kMaxNdim; ++n) c.have_factor[n] = true;
  c.have_hist = false;
  c.launch_status = TGRAD_OK;
  c.profiling = false;
  if (error_pending_on_entry()) return TGRAD_ERR_HIP;
  Plan& p = c.plan;
  if (p.order != TGRAD_ORDER_US_LR) zero_u32(c.stream, c.w<uint32_t>(p.ws_tile_zero), p.ntiles + 1);
  if (t % cfg->refresh_every == 0) {
    rc = do_refresh(&c, grad_dev);
    if (rc != TGRAD_OK) return rc;
  } else {
    // The array is shared by every call on this GPU and may hold another tensor's data: whatever a
    // context keeps in its workspace between a refresh and the steps after it is derived again
    // from the state (the support bitmask, the tile offsets, the factor copies of the fused kernels).
    if (p.k > 0 && p.tile_waves == 0)
      launch_mask_from_indices(c.stream, c.st<int32_t>(p.st_omega), p.k, c.w<uint32_t>(p.ws_mask), p.mask_words);
    launch_tile_offsets(c.stream, c.st<int32_t>(p.st_omega), p.k, p.tile_elems, p.ntiles,
                        c.w<uint32_t>(p.ws_tile_start));
    pack_fused_factor(&c);
  }
  return do_step(&c, weight_dev, grad_dev);
}

int tgrad_get_state(tgrad_ctx* ctx, int what, void* host_out, size_t cap) {
  if (!ctx || !host_out) return TGRAD_ERR_INVALID_ARG;
  Plan& p = ctx->plan;
  if (what == TGRAD_STATE_STEP) {
    if (cap < sizeof(int64_t)) return TGRAD_ERR_TOO_SMALL;
    *static_cast<int64_t*>(host_out) = ctx->t;
    return TGRAD_OK;
  }
  if (what == TGRAD_STATE_INDICES) {
    if (!ctx->have_indices) return TGRAD_ERR_NOT_READY;
    if (cap < (size_t)p.k * 8) return TGRAD_ERR_TOO_SMALL;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return TGRAD_ERR_HIP;
    std::vector<int32_t> tmp((size_t)p.k);
    if (p.k > 0 && hipMemcpy(tmp.data(), ctx->state + p.st_omega, (size_t)p.k * 4, hipMemcpyDeviceToHost) != hipSuccess)
      return TGRAD_ERR_HIP;
    int64_t* o = static_cast<int64_t*>(host_out);
    for (int64_t j = 0; j < p.k; ++j) o[j] = tmp[(size_t)j];
    return TGRAD_OK;
  }
  Item it;
  int rc = locate(ctx, what, &it);
  if (rc != TGRAD_OK) return rc;
  if (it.needs_factor && !ctx->have_factor[it.mode]) return TGRAD_ERR_NOT_READY;
  if (cap < it.bytes) return TGRAD_ERR_TOO_SMALL;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) return TGRAD_ERR_HIP;
  if (it.bytes && hipMemcpy(host_out, it.dev, it.bytes, hipMemcpyDeviceToHost) != hipSuccess) return TGRAD_ERR_HIP;
  if (what >= TGRAD_STATE_FACTOR0 && what < TGRAD_STATE_FACTOR0 + p.N && p.rank[it.mode] < p.shape[it.mode]) {
    // the factor is delivered either way; the status says whether its eigen-solve ran to the end
    int info[2] = {0, 0};
    if (hipMemcpy(info, ctx->ws + p.ws_eig_status + (size_t)4 * it.mode * sizeof(int), sizeof(info),
                  hipMemcpyDeviceToHost) != hipSuccess)
      return TGRAD_ERR_HIP;
    if (info[0] != 0) return TGRAD_ERR_NOT_CONVERGED;
  }
  return TGRAD_OK;
}

int tgrad_check(tgrad_ctx* ctx, int64_t* nonfinite) {
  if (!ctx || !nonfinite) return TGRAD_ERR_INVALID_ARG;
  *nonfinite = -1;
  const Plan& p = ctx->plan;
  if (ctx->cfg.select_rule != TGRAD_SELECT_TOPK_MAG || p.k == 0) return TGRAD_ERR_UNSUPPORTED;
  if (!ctx->have_hist) return TGRAD_ERR_NOT_READY;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) return TGRAD_ERR_HIP;
  // |g|^2 = inf or NaN has all exponent bits set: leading 12-bit digit 0x7F8 or above
  constexpr int kFirst = 0x7F8;
  uint32_t tail[kHistBins - kFirst];
  if (hipMemcpy(tail, ctx->ws + p.ws_hist + (size_t)kFirst * 4, sizeof(tail), hipMemcpyDeviceToHost) != hipSuccess)
    return TGRAD_ERR_HIP;
  int64_t n = 0;
  for (uint32_t v : tail) n += v;
  *nonfinite = n;
  return TGRAD_OK;
}

int tgrad_set_state(tgrad_ctx* ctx, int what, const void* host_in, size_t bytes) {
  if (!ctx || !host_in) return TGRAD_ERR_INVALID_ARG;
  Plan& p = ctx->plan;
  if (what == TGRAD_STATE_STEP) {
    if (bytes != sizeof(int64_t)) return TGRAD_ERR_INVALID_ARG;
    int64_t t = *static_cast<const int64_t*>(host_in);
    if (t < 0) return TGRAD_ERR_INVALID_ARG;
    ctx->t = t;
    return TGRAD_OK;
  }
  if (what == TGRAD_STATE_INDICES) {
    if (bytes != (size_t)p.k * 8) return TGRAD_ERR_INVALID_ARG;
    const int64_t* in = static_cast<const int64_t*>(host_in);
    std::vector<int32_t> tmp((size_t)p.k);
    for (int64_t j = 0; j < p.k; ++j) {
      if (in[j] < 0 || in[j] >= p.I) return TGRAD_ERR_INVALID_ARG;
      if (j > 0 && in[j] <= in[j - 1]) return TGRAD_ERR_INVALID_ARG;
      tmp[(size_t)j] = (int32_t)in[j];
    }
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return TGRAD_ERR_HIP;
    if (p.k > 0) {
      if (hipMemcpy(ctx->state + p.st_omega, tmp.data(), (size_t)p.k * 4, hipMemcpyHostToDevice) != hipSuccess)
        return TGRAD_ERR_HIP;
      Scope sc_(ctx, KID_MASK_FROM_IDX);
      launch_mask_from_indices(ctx->stream, ctx->st<int32_t>(p.st_omega), p.k, ctx->w<uint32_t>(p.ws_mask),
                               p.mask_words);
    }
    {
      Scope sc_(ctx, KID_TILE_OFFSETS);
      launch_tile_offsets(ctx->stream, ctx->st<int32_t>(p.st_omega), p.k, p.tile_elems, p.ntiles,
                          ctx->w<uint32_t>(p.ws_tile_start));
    }
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return TGRAD_ERR_HIP;
    ctx->have_indices = true;
    return check_launch();
  }
  Item it;
  int rc = locate(ctx, what, &it);
  if (rc != TGRAD_OK) return rc;
  if (!it.writable) return TGRAD_ERR_INVALID_ARG;
  if (bytes != it.bytes) return TGRAD_ERR_INVALID_ARG;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) return TGRAD_ERR_HIP;
  if (it.bytes && hipMemcpy(it.dev, host_in, it.bytes, hipMemcpyHostToDevice) != hipSuccess) return TGRAD_ERR_HIP;
  if (it.needs_factor) {
    ctx->have_factor[it.mode] = true;
    if (it.mode == ctx->plan.N - 2) {
      pack_fused_factor(ctx);
      if (hipStreamSynchronize(ctx->stream) != hipSuccess) return TGRAD_ERR_HIP;
      return check_launch();
    }
  }
  return TGRAD_OK;
}

int tgrad_set_profiling(tgrad_ctx* ctx, int enabled) {
  if (!ctx) return TGRAD_ERR_INVALID_ARG;
  int rc = drain_events(ctx);
  if (rc != TGRAD_OK) return rc;
  if (enabled && !ctx->profiling) {
    for (int i = 0; i < KID_COUNT; ++i) {
      ctx->total_ms[i] = 0.;
      ctx->launches[i] = 0;
    }
  }
  ctx->profiling = enabled != 0;
  return TGRAD_OK;
}

int tgrad_get_kernel_times(tgrad_ctx* ctx, const char** names, double* total_ms, int64_t* launches, int cap) {
  if (!ctx || !names || !total_ms || !launches || cap < 0) return TGRAD_ERR_INVALID_ARG;
  int rc = drain_events(ctx);
  if (rc != TGRAD_OK) return rc;
  int n = 0;
  for (int i = 0; i < KID_COUNT && n < cap; ++i) {
    if (ctx->launches[i] == 0) continue;
    names[n] = kKernelNames[i];
    total_ms[n] = ctx->total_ms[i];
    launches[n] = ctx->launches[i];
    ++n;
  }
  return n;
}

int tgrad_calibration_copy(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream) {
  if (!dst_dev || !src_dev || (bytes % 16) || ((uintptr_t)dst_dev % 16) || ((uintptr_t)src_dev % 16))
    return TGRAD_ERR_INVALID_ARG;
  const char* a = static_cast<const char*>(dst_dev);
  const char* b = static_cast<const char*>(src_dev);
  if (a < b + bytes && b < a + bytes) return TGRAD_ERR_INVALID_ARG;
  launch_copy16(static_cast<hipStream_t>(hip_stream), dst_dev, src_dev, (int64_t)(bytes / 16));
  return check_launch();
}

int tgrad_calibration_tile_stream(void* buf_dev, size_t bytes, int tile_bytes, int tiles_per_slab, void* hip_stream,
                                  int64_t* bytes_read) {
  if (!buf_dev || !bytes_read || ((uintptr_t)buf_dev % 16) || tile_bytes < 16 || (tile_bytes % 16) ||
      tile_bytes > 17 * 1024 || tiles_per_slab < 1 || bytes < (size_t)tile_bytes * (size_t)tiles_per_slab)
    return TGRAD_ERR_INVALID_ARG;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return TGRAD_ERR_HIP;
  *bytes_read = launch_tile_stream(static_cast<hipStream_t>(hip_stream), buf_dev, (int64_t)bytes, tile_bytes,
                                   tiles_per_slab, cus);
  return check_launch();
}

int tgrad_calibration_mfma(int kind, int64_t iterations, void* sink_dev, void* hip_stream, double* flops) {
  if ((kind != 0 && kind != 1) || iterations < 1 || iterations > ((int64_t)1 << 32) || !sink_dev || !flops ||
      ((uintptr_t)sink_dev % 4))
    return TGRAD_ERR_INVALID_ARG;
  *flops = launch_mfma_probe(static_cast<hipStream_t>(hip_stream), kind, iterations, static_cast<float*>(sink_dev));
  return check_launch();
}

int tgrad_destroy(tgrad_ctx* ctx) {
  if (!ctx) return TGRAD_ERR_INVALID_ARG;
  (void)drain_events(ctx);
  delete ctx;
  return TGRAD_OK;
}

const char* tgrad_strerror(int status) {
  switch (status) {
    case TGRAD_OK: return "ok";
    case TGRAD_ERR_INVALID_ARG: return "invalid argument";
    case TGRAD_ERR_UNSUPPORTED: return "configuration not supported by this build";
    case TGRAD_ERR_NOT_READY: return "no sparse support / Tucker factors yet (refresh first)";
    case TGRAD_ERR_HIP: return "HIP runtime call or kernel launch failed";
    case TGRAD_ERR_TOO_SMALL: return "host buffer too small";
    case TGRAD_ERR_NOT_CONVERGED: return "eigen-solve of a factor stopped at its sweep limit";
    default: return "unknown status";
  }
}

}  // extern "C"
