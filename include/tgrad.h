/*
 * tgrad.h - C ABI of the TensorGRaD optimizer hot path for AMD MI355X (gfx950).
 *
 * One context (`tgrad_ctx`) serves one complex weight tensor W of an FNO
 * spectral layer and holds the compressed optimizer state of the paper's
 * Algorithm 1 ("Adam with Sparse and Low-Rank Gradient Compression", arxiv
 * 2501.02379): the sparse support Omega, the Tucker factors U^(n), and the Adam
 * moments on the k sparse values and on the Tucker core.
 *
 * Conventions that hold for every call
 *  - Return value: TGRAD_OK (0) or a negative TGRAD_ERR_* code.  Nothing aborts
 *    or throws across this boundary.  `tgrad_strerror` names a code.
 *  - "device pointer" = address in the memory of the GPU that is current when
 *    `tgrad_init` is called; "host pointer" = ordinary process memory.
 *  - The library never allocates or frees device memory.  The caller allocates
 *    `state_dev` and `workspace_dev` with the sizes `tgrad_query_sizes` reports
 *    (256-byte aligned) and keeps both alive until `tgrad_destroy`.
 *  - All device work is enqueued on the one HIP stream given at init.  Neither
 *    `tgrad_step` nor `tgrad_refresh_factors` waits for the device; only
 *    `tgrad_get_state`, `tgrad_set_state` and `tgrad_get_kernel_times` do.
 *  - Every kernel launch is checked where it happens.  A HIP error that is already pending when
 *    `tgrad_step`, `tgrad_step_static` or `tgrad_refresh_factors` is entered belongs to the caller:
 *    the call returns TGRAD_ERR_HIP, launches nothing and leaves the error in place.
 *  - Which kernels serve a configuration is a function of the configuration alone (no environment
 *    switches): matrix-core kernels for the shapes they cover (last-mode rank <= 32 and last extent
 *    >= 2; two modes per pass when the shape allows), one-thread-per-output kernels for the rest.
 *  - A context is used from one host thread at a time.
 *  - Tensors are dense, row-major (last mode fastest).  TGRAD_C64 elements are
 *    interleaved (re, im) float32 pairs (8 bytes); TGRAD_CBF16 elements are
 *    interleaved (re, im) bfloat16 pairs (4 bytes).
 *  - The gradient argument is the ordinary gradient dphi/dW.  Algorithm 1 writes
 *    G = -grad and W <- W + eta * G~; every operation it applies to G is odd, so
 *    this library computes the same W as  W <- W (1 - lr wd) - lr * D(grad).
 */
#ifndef TGRAD_H
#define TGRAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TGRAD_MAX_NDIM 6
#define TGRAD_MAX_HOOI_SWEEPS 64
#define TGRAD_MAX_EIG_SWEEPS 30       /* Jacobi sweeps an eigen-solve may take */
#define TGRAD_MAX_EXTENT 256          /* largest I_n the factor refresh accepts */
#define TGRAD_STATIC_WORKSPACE_BYTES (32u << 20)   /* scratch of tgrad_step_static, per GPU */

typedef struct tgrad_ctx tgrad_ctx;   /* opaque; host memory owned by the library */

enum { TGRAD_C64 = 0, TGRAD_CBF16 = 1 };
enum { TGRAD_SELECT_TOPK_MAG = 0, TGRAD_SELECT_RANDOM = 1 };
enum { TGRAD_ORDER_US_LR = 0, TGRAD_ORDER_LR_US = 1, TGRAD_ORDER_SUM = 2 };

enum {
  TGRAD_OK = 0,
  TGRAD_ERR_INVALID_ARG = -1,   /* null pointer, bad shape/rank/k, misaligned buffer, bad selector */
  TGRAD_ERR_UNSUPPORTED = -2,   /* valid in the paper's terms, but not built (see field comments) */
  TGRAD_ERR_NOT_READY = -3,     /* step or state read before any refresh / factor injection */
  TGRAD_ERR_HIP = -4,           /* a HIP runtime call or kernel launch failed */
  TGRAD_ERR_TOO_SMALL = -5,     /* host buffer smaller than the requested item */
  TGRAD_ERR_NOT_CONVERGED = -6  /* tgrad_get_state of a factor whose eigen-solve stopped at its sweep limit
                                   with rotations still to do (the factor is delivered all the same) */
};

/* Items of `tgrad_get_state` / `tgrad_set_state` (host-side formats in the comments). */
enum {
  TGRAD_STATE_STEP = 0,         /* int64: t, the number of completed steps */
  TGRAD_STATE_INDICES = 1,      /* int64[k]: Omega, ascending row-major linear indices */
  TGRAD_STATE_CORE_M = 2,       /* float32[2*C]: M_L, interleaved complex, C = prod r_n, row-major */
  TGRAD_STATE_CORE_V = 3,       /* float32[C]:   V_L */
  TGRAD_STATE_SPARSE_M = 4,     /* float32[2*k]: M_S, aligned with Omega */
  TGRAD_STATE_SPARSE_V = 5,     /* float32[k]:   V_S */
  TGRAD_STATE_SPARSE_G = 6,     /* float32[2*k]: values gathered at Omega by the last step (read-only) */
  TGRAD_STATE_CORE_G = 7,       /* float32[2*C]: compressed gradient of the last step (read-only) */
  TGRAD_STATE_GRAM0 = 32,       /* + n: float64[2*I_n*I_n] mode-n Gram of the last refresh (read-only) */
  TGRAD_STATE_FACTOR0 = 64,     /* + n: float32[2*I_n*r_n]: U^(n), row-major I_n x r_n, interleaved complex */
  TGRAD_STATE_EIG_INFO0 = 96    /* + n: int32[3] of mode n's last eigen-solve: {1 if it stopped at the sweep limit
                                   else 0, Jacobi sweeps run, 1 if the Jacobi solver ran because the tridiagonal
                                   one declined (close eigenvalues) else 0} (read-only; compressed modes only) */
};

/*
 * Problem statement = the `Require` line of Algorithm 1 (W, eta, alpha, beta1,
 * beta2, rank r, sparsity rho, sparse scale lambda, refresh period T) plus what
 * an implementation must fix (eps, decoupled weight decay, storage types).
 */
typedef struct {
  int32_t ndim;                       /* N, 2..TGRAD_MAX_NDIM */
  int64_t shape[TGRAD_MAX_NDIM];      /* I_n >= 1; I = prod I_n < 2^31; I_n <= TGRAD_MAX_EXTENT */
  int32_t rank[TGRAD_MAX_NDIM];       /* Tucker rank r_n, 1..I_n.  r_n == I_n: the mode is not
                                         compressed (identity factor) */
  int64_t k_sparse;                   /* k = ceil(rho * I), 0..I, computed by the caller exactly */
  int32_t grad_dtype;                 /* TGRAD_C64 or TGRAD_CBF16 */
  int32_t weight_dtype;               /* TGRAD_C64, or TGRAD_CBF16: weights kept in half precision
                                         (section "Mixed precision training"; optimizer states stay
                                         float32): bf16 (re, im) pairs, 4 bytes per element, widened
                                         exactly, updated in float32, rounded once to nearest even */
  float lr;                           /* eta */
  float beta1, beta2, eps;            /* Adam decay rates and epsilon */
  float alpha;                        /* scale of the reconstructed update */
  float lambda;                       /* scale of the sparse part inside it */
  float weight_decay;                 /* decoupled (AdamW) decay; 0 disables */
  int32_t refresh_every;              /* T >= 1: tgrad_step refreshes first when t % T == 0.
                                         0: only tgrad_refresh_factors refreshes */
  int32_t hooi_sweeps;                /* 0 = HOSVD factors (appendix "Implementation": truncated SVD of
                                         each unfolding).  1..TGRAD_MAX_HOOI_SWEEPS: that many HOOI
                                         sweeps after it; a sweep re-solves mode 1, 2, .., N in turn,
                                         each on the residual compressed in every other mode with the
                                         factors as they stand (an updated factor is used at once) */
  int32_t select_rule;                /* how SparseIndices picks Omega (section "Unstructured sparse
                                         gradient tensor"): TGRAD_SELECT_TOPK_MAG = the k entries of
                                         largest |g|^2 (float32), ties to the lower linear index;
                                         TGRAD_SELECT_RANDOM = a uniform random k-subset that depends
                                         only on (select_seed, t at the refresh): the k largest of the
                                         keys fmix32(fmix32(i ^ s0) + s1), fmix32 = MurmurHash3's
                                         32-bit finalizer, s0 = lo32(seed) ^ (t32 * 0x9E3779B9),
                                         s1 = hi32(seed) + t32 + 0x7F4A7C15, t32 = t mod 2^32 */
  uint64_t select_seed;               /* TGRAD_SELECT_RANDOM only */
  int32_t order;                      /* how the two components are composed (paragraph "Residual and
                                         composition"; ablation on sparse / low-rank combinations):
                                         TGRAD_ORDER_US_LR = Algorithm 1: support from G, low rank on G
                                         with the support removed; TGRAD_ORDER_LR_US = low rank on the
                                         full G, the sparse part works on R = G - G~_L (support = top-k
                                         of R at refresh, values = R of the current gradient at the
                                         support every step; the refresh needs one more G-sized
                                         float32 buffer in the workspace); TGRAD_ORDER_SUM = both on
                                         the full G */
  int32_t warm_restart;               /* 0 or 1; 1 needs hooi_sweeps >= 1 (else INVALID_ARG): a refresh
                                         that finds every factor present (from an earlier refresh or
                                         tgrad_set_state) starts its sweeps from those factors instead
                                         of from HOSVD (the warm restart of the same appendix) */
  int32_t eig_max_sweeps;             /* which eigen-solver the refresh uses for extents up to 128:
                                         0 = Householder tridiagonalisation + bisection + inverse iteration,
                                         and cyclic Jacobi (up to TGRAD_MAX_EIG_SWEEPS sweeps) only for a matrix
                                         whose leading eigenvalues are too close for inverse iteration;
                                         1..TGRAD_MAX_EIG_SWEEPS = cyclic Jacobi with that many sweeps at most
                                         for every solve (extents above 128 always use Jacobi).  A Jacobi solve
                                         that uses its sweeps up is reported by tgrad_get_state (NOT_CONVERGED) */
} tgrad_config;

/*
 * Bytes of device memory a context needs.  Host-only, touches no GPU.
 *  cfg             host pointer, read only.
 *  state_bytes     host pointer, out: persistent optimizer state (Omega as int32, M_S, V_S, M_L,
 *                  V_L, U^(n); the quantity the paper's memory model counts).
 *  workspace_bytes host pointer, out: scratch that carries nothing from one step to the next
 *                  except kernel-ready copies of the factors and the support bitmask.
 * Errors: INVALID_ARG, UNSUPPORTED.
 */
int tgrad_query_sizes(const tgrad_config* cfg, size_t* state_bytes, size_t* workspace_bytes);

/*
 * Create a context (Algorithm 1, the initialisation lines: t <- 0, all moments <- 0).
 *  out            host pointer, receives the context.
 *  cfg            host pointer, copied.
 *  state_dev      device pointer, >= state_bytes, 256-byte aligned; zeroed asynchronously here.
 *  workspace_dev  device pointer, >= workspace_bytes, 256-byte aligned.
 *  hip_stream     a hipStream_t (NULL = the default stream); every later call enqueues on it.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP.
 */
int tgrad_init(tgrad_ctx** out, const tgrad_config* cfg, void* state_dev, void* workspace_dev,
               void* hip_stream);

/*
 * Algorithm 1, the `t mod T = 0` branch, for cfg.order == TGRAD_ORDER_US_LR:
 * Omega <- SparseIndices(G, rho, cfg.select_rule); R_L <- G - Sparse(G, Omega);
 * {U^(n)} <- TuckerFactors(R_L, r): HOSVD (eigenvectors of the r_n largest eigenvalues of each mode-n
 * Gram matrix R_L(n) R_L(n)^H, descending, every column multiplied by the unit phase that makes its
 * largest-modulus entry real and positive), then cfg.hooi_sweeps HOOI sweeps (from the factors in
 * place instead of from HOSVD when cfg.warm_restart applies).  The two other composition orders
 * take the factors from the full G and (TGRAD_ORDER_LR_US) the support from G - G~_L; see cfg.order.
 * Top-k order: (|g|^2 descending, linear index ascending), |g|^2 evaluated in float32 as
 * fl(fl(re*re) + fl(im*im)).  Touches neither the moments nor t.
 *  grad_dev   device pointer to G (cfg.grad_dtype), read only.
 * Errors: INVALID_ARG, HIP.
 */
int tgrad_refresh_factors(tgrad_ctx* ctx, const void* grad_dev);

/*
 * One pass of Algorithm 1's loop body on (W, G): refresh first if cfg.refresh_every > 0 and
 * t % refresh_every == 0; g_S <- G[Omega]; g_L <- (G with Omega zeroed) x_1 U1^H ... x_N UN^H;
 * AdamUpdate on g_S with (M_S, V_S) and on g_L with (M_L, V_L), tau = t + 1 in the bias
 * correction, N = (M / (1 - beta1^tau)) / (sqrt(V / (1 - beta2^tau)) + eps), V from |x|^2;
 * D <- alpha * (N_L x_1 U1 ... x_N UN); D[Omega] += lambda * N_S;
 * W <- W (1 - lr wd) - lr D; t <- t + 1.
 *  weight_dev  device pointer to W (layout per cfg.weight_dtype), updated in place.
 *  grad_dev    device pointer to G (cfg.grad_dtype), read only, must not alias W.
 * Errors: INVALID_ARG, NOT_READY (refresh_every == 0 and no refresh yet), HIP.
 */
int tgrad_step(tgrad_ctx* ctx, void* weight_dev, const void* grad_dev);

/*
 * tgrad_step for callers that cannot allocate device memory and cannot hold a context: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It does what
 * `tgrad_step` does for a context at step count t (refresh first when t % cfg.refresh_every == 0,
 * then the loop body), but allocates nothing, neither on the device nor on the host: there is no
 * context, and the scratch that `workspace_dev` provides elsewhere is a fixed array inside the
 * library, TGRAD_STATIC_WORKSPACE_BYTES per GPU, which every GPU that runs the library holds until
 * the process ends.  A configuration whose `tgrad_query_sizes` workspace exceeds that size is
 * rejected with TGRAD_ERR_UNSUPPORTED and nothing is launched.
 *  cfg         host pointer; refresh_every must be >= 1 (INVALID_ARG otherwise).
 *  state_dev   device pointer, >= state_bytes of `tgrad_query_sizes`, 256-byte aligned: the optimizer
 *              state (Omega, M_S, V_S, M_L, V_L, U^(n)).  The caller zero-fills it before the call
 *              with t = 0 and passes the same buffer, untouched, to the calls with t = 1, 2, ...; a
 *              call with t % refresh_every != 0 on a state that no earlier call has refreshed is
 *              not detected.
 *  t           the number of steps this state has taken so far.
 *  weight_dev, grad_dev  as for `tgrad_step`.
 *  hip_stream  stream to enqueue on (NULL = the default stream).  Does not wait.
 * All calls on one GPU share that GPU's array, which keeps the last call's contents: every call
 * rebuilds what it reads from there, and calls that overlap in time on one GPU (two streams, two
 * threads) race.  The device must be the current one.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP.
 */
int tgrad_step_static(const tgrad_config* cfg, void* state_dev, int64_t t, void* weight_dev,
                      const void* grad_dev, void* hip_stream);

/*
 * Copy one state item to the host (waits for the stream first).
 *  what      a TGRAD_STATE_* selector (FACTOR0 + n / GRAM0 + n for mode n).
 *  host_out  host pointer, receives the item in the format listed at the selector.
 *  cap       bytes available at host_out.
 * Errors: INVALID_ARG, TOO_SMALL, NOT_READY (indices/factors before any refresh), HIP.
 */
int tgrad_get_state(tgrad_ctx* ctx, int what, void* host_out, size_t cap);

/*
 * Non-finite gradient entries seen by the last refresh (waits for the stream).  The top-k selection
 * already builds a histogram of the leading bits of |g|^2 for every refresh; the entries whose
 * |g|^2 is inf or NaN (a non-finite part, or a magnitude above 1.8e19) are its top bins, so this
 * costs no extra pass over the gradient.  Algorithm 1 is undefined on such a gradient.
 *  nonfinite  host pointer, out: their number.
 * Errors: INVALID_ARG; UNSUPPORTED (rand-k selection or k_sparse == 0: no such histogram exists);
 *         NOT_READY (no refresh yet); HIP.
 */
int tgrad_check(tgrad_ctx* ctx, int64_t* nonfinite);

/*
 * Overwrite one state item from the host (checkpoint restore, or injecting externally computed
 * factors / support).  Read-only selectors are rejected.  INDICES must be strictly ascending and
 * within [0, I); setting INDICES and every FACTOR marks the context ready.  Waits for the stream.
 * Errors: INVALID_ARG, HIP.
 */
int tgrad_set_state(tgrad_ctx* ctx, int what, const void* host_in, size_t bytes);

/*
 * Per-kernel timing with HIP events on the context's stream (for roofline reports).
 * `tgrad_set_profiling(ctx, 1)` makes later calls bracket every kernel launch with events;
 * `tgrad_get_kernel_times` waits for the stream and returns, for up to `cap` kernels, the name
 * (pointer to a static string), the summed duration in milliseconds and the launch count since
 * profiling was last switched on.  Returns the number of kernels written (>= 0) or an error.
 */
int tgrad_set_profiling(tgrad_ctx* ctx, int enabled);
int tgrad_get_kernel_times(tgrad_ctx* ctx, const char** names, double* total_ms, int64_t* launches,
                           int cap);

/*
 * Plain device-to-device copy kernel of a known size, for calibrating hardware counters: a
 * profiler's HBM read / write counters for this launch correspond to exactly `bytes` read and
 * `bytes` written, which fixes the scale of the same counters on the optimizer's kernels.
 *  dst_dev, src_dev  device pointers, 16-byte aligned, non-overlapping, `bytes` long each.
 *  bytes             a multiple of 16.
 *  hip_stream        stream to enqueue on (NULL = the default stream).  Does not wait.
 * Errors: INVALID_ARG, HIP.
 */
int tgrad_calibration_copy(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream);

/*
 * The memory access pattern of the weight-update kernel without its arithmetic, for calibrating that kernel's
 * bandwidth fraction: every wavefront owns a tile of `tile_bytes`, loads all of it and then stores it back in
 * place unchanged; wavefronts take slabs of `tiles_per_slab` consecutive tiles.  (The plain copy above moves
 * the same bytes with fewer concurrent streams and reaches a higher rate; this is the ceiling of the pattern
 * that a kernel with one tile per wavefront has.)
 *  buf_dev         device pointer, 16-byte aligned, `bytes` long; its contents are rewritten with themselves.
 *  bytes           at least tile_bytes * tiles_per_slab; whole slabs are moved, a remainder is left alone.
 *  tile_bytes      a multiple of 16, at most 17408 (the update kernel's tile: 32 rows of the last mode).
 *  tiles_per_slab  >= 1 (the update kernel: extent of mode N-1 / 32).
 *  hip_stream      stream to enqueue on (NULL = the default stream).  Does not wait.
 *  bytes_read      host pointer: receives the bytes the launch reads (it writes as many).
 * Errors: INVALID_ARG, HIP.
 */
int tgrad_calibration_tile_stream(void* buf_dev, size_t bytes, int tile_bytes, int tiles_per_slab, void* hip_stream,
                                  int64_t* bytes_read);

/*
 * Register-resident matrix-core loop over the whole chip, for calibrating the matrix-core fractions that
 * are reported for the projection and Gram kernels: what the hardware delivers with no memory traffic at all.
 *  kind        0 = the float32 instruction of the projection kernels (32 x 32 x 2), 1 = the float64
 *              instruction of the Gram kernels (16 x 16 x 4).
 *  iterations  loop length per wavefront, >= 1 (each iteration issues four matrix instructions).
 *  sink_dev    device pointer to at least 4 writable bytes, 4-byte aligned (never written in practice: it
 *              keeps the loop from being optimised away).
 *  hip_stream  stream to enqueue on (NULL = the default stream).  Does not wait.
 *  flops       host pointer: receives the floating-point operations of the launch (2 per multiply-add);
 *              divide by the launch's duration, measured by the caller on that stream.
 * Errors: INVALID_ARG, HIP.
 */
int tgrad_calibration_mfma(int kind, int64_t iterations, void* sink_dev, void* hip_stream, double* flops);

/* Release the context (host memory only; device buffers stay the caller's). */
int tgrad_destroy(tgrad_ctx* ctx);

/* Static description of a status code. */
const char* tgrad_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* TGRAD_H */
