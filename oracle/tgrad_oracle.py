"""CPU oracle for the TensorGRaD optimizer step (TEST INFRASTRUCTURE ONLY).

This file is the slow, plain definition of what the GPU library must compute.
It is numpy in float64 / complex128 throughout, except the selection key,
which the method's tie-break forces into float32 (see `selection_key`).  It
shares no code with the HIP path and must never be imported by it: only the
tests, the smoke check and the bench's `cpu_baseline` leg may use it.

What it follows, in the paper's notation (arxiv 2501.02379):

* Algorithm 1 ("Adam with Sparse and Low-Rank Gradient Compression"): the
  refresh branch (`t mod T = 0`: SparseIndices, residual R_L = G - Sparse(G,
  Omega), TuckerFactors) and the per-step body (Sparse gather, low-rank
  compression with the conjugate-transposed factors, AdamUpdate on both
  compressed parts, reconstruction scaled by alpha, scatter-add of lambda times
  the sparse part, weight update, t <- t + 1).
* The appendix algorithm "Adam with low-rank tensor decomposition" for the body
  of AdamUpdate (first moment, second moment from |R * conj(R)|, bias
  correction, N = M / (sqrt(V) + eps)).
* Section "Unstructured sparse gradient tensor": k = ceil(rho * I), COO
  index/value pairs, Omega fixed between refreshes, values re-read every step.
* Section "Low-rank gradient tensor decomposition": orthonormal factors,
  compression G x_n U^(n)H, reconstruction with U^(n).
* Appendix "Tensor Operations and Notation": mode-k unfolding and mode-k
  product definitions.
* Appendix remark "Real-Valued Analysis": for complex tensors every transpose is
  a conjugate transpose.
* Appendix "Implementation" (HOI): factors start from the truncated SVD of each
  mode-n unfolding (HOSVD); optional refinement sweeps (HOOI).

Readings taken where the paper is silent or inconsistent (each also listed in
the design notes of this repository):

* V is real (it is built from |R conj R|), although Algorithm 1 declares it
  complex.
* Bias correction uses tau = t + 1 (t starts at 0 and `t mod T` uses that t, so
  the very first step refreshes; 1 - beta^0 would divide by zero).
* M_S, V_S are length-k vectors aligned with Omega stored in ascending linear
  (row-major) index; the shape Algorithm 1 prints for them belongs to the
  structured-sparsity variant.
* Moments are NOT reset when Omega or the factors change (Algorithm 1 shows no
  reset).
* Top-k magnitude selection orders entries by (|g|^2 descending, linear index
  ascending); |g|^2 is evaluated in float32 as fl(fl(re*re) + fl(im*im)).
* TuckerFactors = HOSVD: eigenvectors of the r_n largest eigenvalues of the
  mode-n Gram matrix, eigenvalue-descending, each column multiplied by the unit
  phase that makes its largest-modulus entry (lowest row on ties) real and
  positive.  r_n = I_n selects the identity (the mode is not compressed).
* The gradient argument is the ordinary gradient dphi/dW; the paper's
  G = -grad and W <- W + eta * G~ is the same update because every operation
  applied to G is odd.
* AdamW decay is decoupled: W <- W (1 - lr wd) - lr * D (pinned to torch.optim.AdamW).
* The appendix algorithm "Adam with low-rank tensor decomposition" assigns the
  bias-corrected moments to the same symbols M_t, V_t it carries to the next
  step.  Read literally that would divide the stored moments by (1 - beta^t)
  again at every step; it is read here as standard Adam: the corrected values
  are temporaries of the step, the stored moments are the raw ones (this is what
  torch.optim.Adam does, which pins `adam_update` over several steps).
* Composition orders other than Algorithm 1's (paragraph "Residual and
  composition", ablation on combinations): "lr_us" compresses the full gradient
  to low rank first and gives the sparse part the residual of that low-rank
  approximation (support = top-k of the residual at refresh, values = the
  residual of the CURRENT gradient at the support every step); "sum" applies
  both to the full gradient.  For the top-k key the residual is rounded to
  complex64 first (the key is defined on float32 parts).
* Half-precision weights are bf16 (re, im) pairs without a full-precision copy:
  each step widens them, applies the update and rounds the result once, to
  nearest even.  The paper says only that weights are kept in half precision.
* Uniform random selection (rand-k) draws its subset from a counter-based integer
  hash of (index, seed, step count at the refresh); see `random_keys`.  The
  paper does not say how the subset is drawn.

* HOOI refinement (appendix "Implementation": the factors are refined iteratively
  and a warm restart reuses the previous ones): a sweep re-solves mode 1, 2, ..., N
  in turn, each on the tensor compressed in every OTHER mode with the factors as
  they stand at that moment (an updated factor is used at once by the modes after
  it); the sweep count is a parameter.  Warm restart: from the second refresh on,
  the sweeps start from the factors in use instead of from HOSVD.

Parity pins for every function below live in tests/test_oracle_*.py.  The HOOI
refinement sweeps (`hooi_sweeps > 0`) are "parity unpinned" beyond monotone core
energy, the exact-low-rank fixed point and the one-sweep closed form on an
order-2 tensor: the paper gives no sweep count.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from fractions import Fraction
from typing import List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------
# sizes
# --------------------------------------------------------------------------
def sparse_count(rho: Fraction, numel: int) -> int:
    """k = ceil(rho * I), section "Unstructured sparse gradient tensor".

    rho is an exact fraction so no float rounding enters the ceiling."""
    rho = Fraction(rho)
    return int(-((-rho.numerator * numel) // rho.denominator))


def optimizer_state_params_tucker(shape: Sequence[int], ranks: Sequence[int]) -> int:
    """Parameter count of the Tucker optimizer state as the paper's worked
    example counts it (appendix "Memory Savings Analysis"): core entries plus
    one I_n x r_n factor per mode (the example's 2(16)(64) + 2(16)(128) are the
    two channel modes and the two Fourier modes)."""
    core = 1
    for r in ranks:
        core *= int(r)
    return core + sum(int(r) * int(i) for i, r in zip(shape, ranks))


def optimizer_state_params_matrix(rows: int, cols: int, rank: int) -> int:
    """Matrix-GaLore count of the same worked example: r^2 (rows^2 + cols^2)."""
    return rank * rank * (rows * rows + cols * cols)


# --------------------------------------------------------------------------
# input decoding (exact)
# --------------------------------------------------------------------------
def bf16_pairs_to_complex(raw: np.ndarray) -> np.ndarray:
    """(…, 2) uint16 bf16 bit patterns (re, im) -> complex128, exactly.

    A bf16 is the upper half of a float32, so widening is a 16-bit shift."""
    raw = np.asarray(raw, dtype=np.uint16)
    f = (raw.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return f[..., 0].astype(np.float64) + 1j * f[..., 1].astype(np.float64)


def _as_c64_pairs(G: np.ndarray) -> np.ndarray:
    """Return the float32 (re, im) pairs of a gradient given as complex64 or as
    bf16 pairs (uint16 with a trailing axis of 2)."""
    G = np.asarray(G)
    if G.dtype == np.uint16:
        return (G.astype(np.uint32) << np.uint32(16)).view(np.float32)
    if G.dtype != np.complex64:
        raise TypeError("gradient must be complex64 or uint16 bf16 pairs")
    return np.ascontiguousarray(G).view(np.float32).reshape(G.shape + (2,))


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Real float64 values -> bf16 bit patterns (uint16), round to nearest, ties to even.

    bf16 = 1 sign, 8 exponent, 7 stored fraction bits: a normal number x = m 2^e with
    0.5 <= |m| < 1 lies on a grid of spacing 2^(e-8); below the smallest normal (2^-126) the
    spacing stays 2^-133.  numpy's rint rounds halves to even, which on that grid is the
    required tie rule.  Values beyond the largest finite bf16 become infinities."""
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    e = np.maximum(e, -125)
    q = np.ldexp(1.0, e - 8)
    y = np.rint(x / q) * q
    y = np.where(np.abs(y) > 3.3895313892515355e38, np.copysign(np.inf, y), y)   # (2 - 2^-7) 2^127
    f = y.astype(np.float32)                                 # exact: every bf16 is a float32
    bits = (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    return np.where(np.isnan(x), np.uint16(0x7FC0), bits).astype(np.uint16)


def complex_to_bf16_pairs(Z: np.ndarray) -> np.ndarray:
    """complex128 -> (..., 2) uint16 bf16 bit patterns (re, im), each part rounded to nearest even."""
    Z = np.asarray(Z, dtype=np.complex128)
    return np.stack([round_to_bf16_bits(Z.real), round_to_bf16_bits(Z.imag)], axis=-1)


def to_complex128(G: np.ndarray) -> np.ndarray:
    p = _as_c64_pairs(G)
    return p[..., 0].astype(np.float64) + 1j * p[..., 1].astype(np.float64)


# --------------------------------------------------------------------------
# sparse part
# --------------------------------------------------------------------------
def selection_key(G: np.ndarray) -> np.ndarray:
    """|g|^2 in float32: fl(fl(re*re) + fl(im*im)), one rounding per operation,
    no fused multiply-add.  Flat, row-major."""
    p = _as_c64_pairs(G).reshape(-1, 2)
    re = p[:, 0]
    im = p[:, 1]
    rr = np.multiply(re, re, dtype=np.float32)
    ii = np.multiply(im, im, dtype=np.float32)
    return np.add(rr, ii, dtype=np.float32)


def sparse_indices(G: np.ndarray, k: int) -> np.ndarray:
    """SparseIndices(G, rho, top-k): the k entries first in the order
    (key descending, linear index ascending), returned ascending (int64)."""
    key = selection_key(G)
    if k < 0 or k > key.size:
        raise ValueError("k out of range")
    # stable sort of the negated key: equal keys keep ascending index order
    order = np.argsort(-key, kind="stable")
    return np.sort(order[:k]).astype(np.int64)


# --------------------------------------------------------------------------
# uniform random support (rand-k)
# --------------------------------------------------------------------------
# The paper names uniform random selection of the k entries as an alternative to top-k
# (section "Unstructured sparse gradient tensor"; the ablation on selection strategies) and says
# nothing about the sampler.  Reading used here: every linear index i gets a pseudo-random 32-bit
# key that depends only on (i, seed, t) -- t the step count at the refresh -- and the support is
# the k indices with the largest keys.  The key map is a bijection of the 32-bit integers, so the
# keys of distinct indices differ and the subset is what a random permutation of the indices
# would give.  The mixing function is the 32-bit finalizer of MurmurHash3 (a public-domain,
# published integer hash), applied twice around the two seed words.
_M32 = 0xFFFFFFFF


def _fmix32(x: np.ndarray) -> np.ndarray:
    x = x.astype(np.uint64)                     # products below stay under 2^64
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x85EBCA6B)) & np.uint64(_M32)
    x ^= x >> np.uint64(13)
    x = (x * np.uint64(0xC2B2AE35)) & np.uint64(_M32)
    x ^= x >> np.uint64(16)
    return x


def random_key_words(seed: int, t: int):
    """The two 32-bit words (s0, s1) the keys of one refresh are built from."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    t32 = int(t) & _M32
    s0 = (seed & _M32) ^ ((t32 * 0x9E3779B9) & _M32)
    s1 = ((seed >> 32) + t32 + 0x7F4A7C15) & _M32
    return s0, s1


def random_keys(numel: int, seed: int, t: int) -> np.ndarray:
    """key(i) = fmix32(fmix32(i xor s0) + s1) for i = 0 .. numel-1 (uint32)."""
    s0, s1 = random_key_words(seed, t)
    i = np.arange(numel, dtype=np.uint64)
    a = _fmix32(i ^ np.uint64(s0))
    return _fmix32((a + np.uint64(s1)) & np.uint64(_M32)).astype(np.uint32)


def sparse_indices_random(numel: int, k: int, seed: int, t: int) -> np.ndarray:
    """SparseIndices(., rho, rand-k): the k indices first in the order (key descending, linear
    index ascending) of the pseudo-random keys, returned ascending (int64)."""
    if k < 0 or k > numel:
        raise ValueError("k out of range")
    key = random_keys(numel, seed, t)
    order = np.argsort(-key.astype(np.int64), kind="stable")
    return np.sort(order[:k]).astype(np.int64)


def sparse_gather(Gc: np.ndarray, omega: np.ndarray) -> np.ndarray:
    """Sparse(G, Omega): the values at Omega (COO values, Omega order)."""
    return np.ascontiguousarray(Gc).reshape(-1)[omega].copy()


def remove_sparse(Gc: np.ndarray, omega: np.ndarray) -> np.ndarray:
    """G - Sparse(G, Omega): G with the entries at Omega set to zero."""
    X = np.array(Gc, order="C", copy=True)      # C order: reshape(-1) below is a view
    X.reshape(-1)[omega] = 0.0
    return X


# --------------------------------------------------------------------------
# tensor algebra
# --------------------------------------------------------------------------
def unfold(X: np.ndarray, n: int) -> np.ndarray:
    """A mode-n unfolding: rows indexed by i_n, columns by all other indices.

    The column order here is numpy's (remaining modes in row-major order), not
    the order of the paper's unfolding definition; everything computed from it
    in this file (the Gram matrix) does not depend on the column order."""
    return np.moveaxis(X, n, 0).reshape(X.shape[n], -1)


def mode_product(X: np.ndarray, A: np.ndarray, n: int) -> np.ndarray:
    """X x_n A for A of shape (J, I_n): out[.., j, ..] = sum_i X[.., i, ..] A[j, i]."""
    if A.shape[1] != X.shape[n]:
        raise ValueError("mode_product: extent mismatch")
    out = np.tensordot(A, X, axes=(1, n))       # mode n lands on axis 0
    return np.moveaxis(out, 0, n)


def compress(X: np.ndarray, U: Sequence[np.ndarray]) -> np.ndarray:
    """X x_1 U1^H ... x_N UN^H."""
    R = X
    for n, Un in enumerate(U):
        R = mode_product(R, Un.conj().T, n)
    return R


def reconstruct(C: np.ndarray, U: Sequence[np.ndarray]) -> np.ndarray:
    """C x_1 U1 ... x_N UN."""
    D = C
    for n, Un in enumerate(U):
        D = mode_product(D, Un, n)
    return D


def mode_gram(X: np.ndarray, n: int) -> np.ndarray:
    """A_n = X_(n) X_(n)^H, Hermitian I_n x I_n."""
    Xn = unfold(X, n)
    return Xn @ Xn.conj().T


def _phase_normalise(V: np.ndarray) -> np.ndarray:
    V = V.copy()
    for c in range(V.shape[1]):
        col = V[:, c]
        p = int(np.argmax(np.abs(col)))          # first maximum = lowest row
        a = col[p]
        if a != 0:
            V[:, c] = col * (np.conj(a) / np.abs(a))
    return V


def top_eigvecs(A: np.ndarray, r: int) -> np.ndarray:
    """Eigenvectors of the r largest eigenvalues of Hermitian A, descending,
    phase-normalised; r == order of A returns the identity."""
    n = A.shape[0]
    if r == n:
        return np.eye(n, dtype=np.complex128)
    w, V = np.linalg.eigh(A)                    # ascending
    V = V[:, ::-1][:, :r]
    return _phase_normalise(V)


def tucker_factors(X: np.ndarray, ranks: Sequence[int], hooi_sweeps: int = 0,
                   init: Optional[Sequence[np.ndarray]] = None) -> List[np.ndarray]:
    """TuckerFactors(R_L, r).  HOSVD (left singular vectors of each unfolding,
    obtained as Gram eigenvectors), then `hooi_sweeps` HOOI sweeps in which mode
    n is re-solved on X compressed in every other mode.  `init` (a previous set
    of factors) replaces the HOSVD start: the warm restart."""
    N = X.ndim
    if init is None:
        U = [top_eigvecs(mode_gram(X, n), ranks[n]) for n in range(N)]
    else:
        U = [u.copy() for u in init]
    for _ in range(hooi_sweeps):
        for n in range(N):
            Y = X
            for m in range(N):
                if m != n:
                    Y = mode_product(Y, U[m].conj().T, m)
            U[n] = top_eigvecs(mode_gram(Y, n), ranks[n])
    return U


# --------------------------------------------------------------------------
# Adam in a compressed space
# --------------------------------------------------------------------------
def adam_update(x: np.ndarray, M: np.ndarray, V: np.ndarray, beta1: float,
                beta2: float, tau: int, eps: float):
    """AdamUpdate: returns (N, M_new, V_new) for compressed gradient x.

    M complex, V real; tau >= 1 is the 1-based step used for bias correction."""
    M = beta1 * M + (1.0 - beta1) * x
    V = beta2 * V + (1.0 - beta2) * (x * np.conj(x)).real
    Mhat = M / (1.0 - beta1 ** tau)
    Vhat = V / (1.0 - beta2 ** tau)
    return Mhat / (np.sqrt(Vhat) + eps), M, V


# --------------------------------------------------------------------------
# the optimizer
# --------------------------------------------------------------------------
@dataclass
class Hyper:
    ranks: Sequence[int]
    k: int
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    alpha: float = 1.0
    lam: float = 1.0
    weight_decay: float = 0.0
    T: int = 1                 # refresh when t % T == 0; 0 = only on request
    hooi_sweeps: int = 0
    warm_restart: bool = False  # with hooi_sweeps >= 1: later refreshes start from the current factors
    order: str = "us_lr"       # composition: "us_lr" (Algorithm 1), "lr_us", or "sum"
    select_rule: str = "topk"  # "topk" (magnitude) or "randk" (uniform random subset)
    select_seed: int = 0       # rand-k only


@dataclass
class State:
    shape: Sequence[int]
    hyper: Hyper
    t: int = 0
    omega: Optional[np.ndarray] = None
    U: Optional[List[np.ndarray]] = None
    M_L: np.ndarray = field(default=None)
    V_L: np.ndarray = field(default=None)
    M_S: np.ndarray = field(default=None)
    V_S: np.ndarray = field(default=None)

    def __post_init__(self):
        r = tuple(int(x) for x in self.hyper.ranks)
        if len(r) != len(self.shape):
            raise ValueError("one rank per mode")
        for i, x in zip(self.shape, r):
            if not (1 <= x <= i):
                raise ValueError("rank out of range")
        self.M_L = np.zeros(r, dtype=np.complex128)
        self.V_L = np.zeros(r, dtype=np.float64)
        self.M_S = np.zeros(self.hyper.k, dtype=np.complex128)
        self.V_S = np.zeros(self.hyper.k, dtype=np.float64)


def _select(st: State, X: np.ndarray) -> np.ndarray:
    """SparseIndices on X (complex64 or bf16 pairs) by the configured rule."""
    if st.hyper.select_rule == "randk":
        return sparse_indices_random(int(np.prod(st.shape)), st.hyper.k, st.hyper.select_seed, st.t)
    if st.hyper.select_rule == "topk":
        return sparse_indices(X, st.hyper.k)
    raise ValueError("unknown selection rule")


def refresh(st: State, G: np.ndarray) -> None:
    """The `t mod T = 0` branch.  Touches neither moments nor t.

    order "us_lr" is Algorithm 1: the support comes from G, the factors from G with the support
    removed.  The paragraph "Residual and composition" and the ablation on sparse / low-rank
    combinations define the two other orders: "lr_us" - the first component (low rank) sees the
    full gradient and the second (sparse) the residual R = G - G~_L of the first; "sum" - both see
    the full gradient and their outputs are added."""
    h = st.hyper
    if h.order not in ("us_lr", "lr_us", "sum"):
        raise ValueError("unknown composition order")
    if h.warm_restart and h.hooi_sweeps < 1:
        raise ValueError("warm restart needs at least one HOOI sweep")
    Gc = to_complex128(G)
    init = st.U if (h.warm_restart and st.U is not None) else None
    if h.order == "us_lr":
        st.omega = _select(st, G)
        st.U = tucker_factors(remove_sparse(Gc, st.omega), h.ranks, h.hooi_sweeps, init)
    elif h.order == "sum":
        st.omega = _select(st, G)
        st.U = tucker_factors(Gc, h.ranks, h.hooi_sweeps, init)
    else:
        st.U = tucker_factors(Gc, h.ranks, h.hooi_sweeps, init)
        R = Gc - reconstruct(compress(Gc, st.U), st.U)
        st.omega = _select(st, R.astype(np.complex64))       # the key is formed from float32 parts


def step(st: State, W: np.ndarray, G: np.ndarray) -> np.ndarray:
    """One pass of Algorithm 1's loop body; returns W_{t+1} (complex128).

    Weights stored in half precision (section "Mixed precision training": weights, activations and
    gradients in half precision, optimizer states in full precision): W given as bf16 pairs
    (uint16, trailing axis 2) is widened exactly, updated as below, and returned rounded ONCE to
    bf16 pairs (nearest even) - there is no full-precision copy of the weights."""
    if np.asarray(W).dtype == np.uint16:
        return complex_to_bf16_pairs(step(st, bf16_pairs_to_complex(W), G))
    h = st.hyper
    if h.T > 0 and st.t % h.T == 0:
        refresh(st, G)
    if st.omega is None:
        raise RuntimeError("step before any refresh")
    Gc = to_complex128(G)
    W = np.asarray(W, dtype=np.complex128)

    if h.order == "us_lr":
        g_S = sparse_gather(Gc, st.omega)                   # sparse tensor, current step
        g_L = compress(remove_sparse(Gc, st.omega), st.U)   # low-rank compression of the rest
    elif h.order == "sum":
        g_S = sparse_gather(Gc, st.omega)                   # both components see the full gradient
        g_L = compress(Gc, st.U)
    else:                                                   # lr_us: the sparse part sees the residual
        g_L = compress(Gc, st.U)
        g_S = sparse_gather(Gc - reconstruct(g_L, st.U), st.omega)

    tau = st.t + 1
    n_S, st.M_S, st.V_S = adam_update(g_S, st.M_S, st.V_S, h.beta1, h.beta2, tau, h.eps)
    n_L, st.M_L, st.V_L = adam_update(g_L, st.M_L, st.V_L, h.beta1, h.beta2, tau, h.eps)

    D = np.ascontiguousarray(h.alpha * reconstruct(n_L, st.U))   # low-rank part first
    D.reshape(-1)[st.omega] += h.lam * n_S                  # sparse values added into it (view)
    W_new = W * (1.0 - h.lr * h.weight_decay) - h.lr * D
    st.t += 1
    return W_new


def dense_complex_adam_step(W, G, M, V, t, lr, beta1, beta2, eps, weight_decay=0.0):
    """Plain complex Adam on the full tensor (what the method must reduce to
    with k = I, or with every rank full and k = 0).  Returns (W, M, V)."""
    Gc = to_complex128(G)
    n, M, V = adam_update(Gc, M, V, beta1, beta2, t + 1, eps)
    return W * (1.0 - lr * weight_decay) - lr * n, M, V
