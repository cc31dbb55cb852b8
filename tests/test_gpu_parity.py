"""GPU-vs-oracle parity of the HIP library, through its C ABI.

Bars (from the benchmark spec): sparse indices bit-exact; updated weights within 1e-4 relative
(Frobenius) after 10 steps; factors within 1e-3 as subspace projectors.  On top of that
(helpers.check_parity) the update W_t - W_0 itself within 1e-4 relative, so that the check is
sensitive to the optimizer and not to W_0, every entry of it within 1e-2 lr sqrt(steps), and the
four Adam moment arrays entry by entry.
"""
import numpy as np
import pytest

from oracle import tgrad_oracle as O
from paper_2501_02379_amd import synth
from paper_2501_02379_amd import tgrad as T
from helpers import (projector_distance, rel_err, run_both, make_gpu_ctx, run_both_bf16_weights, bf16_ordinal,
                     check_parity)

pytestmark = pytest.mark.gpu

PROJ_TOL = 1e-3


def _announce(*a):
    print("[case]", *a, flush=True)


# ------------------------------------------------------------------ selection
SEL_CASES = [
    ((3, 4, 2), 1, "c64"), ((5, 7), 2, "c64"), ((7, 5, 3, 2), 3, "c64"), ((16, 16, 8, 5), 4, "c64"),
    ((6, 5, 4), 11, "cbf16"), ((33, 17, 9), 5, "c64"), ((65, 64, 33), 6, "c64"), ((32, 31, 17, 3), 7, "cbf16"),
]


@pytest.mark.parametrize("shape,seed,dt", SEL_CASES)
def test_sparse_indices_bit_exact(shape, seed, dt):
    g = synth.small_case(shape, seed, outlier_frac=(1, 50), dtype=dt, ties=True)
    I = int(np.prod(shape))
    gd = T.to_device_grad(g)
    for k in sorted(set([0, 1, 2, I // 100 + 1, I // 7, I // 2, I - 1, I])):
        _announce("select", shape, dt, "k=", k)
        ctx = make_gpu_ctx(T, shape, [1] * len(shape), k, grad_dtype=T.TGRAD_CBF16 if dt == "cbf16" else 0,
                           refresh_every=0)
        ctx.tgrad_refresh_factors(gd)
        got = ctx.tgrad_get_state(T.STATE_INDICES)
        want = O.sparse_indices(g, k)
        assert got.dtype == np.int64 and np.array_equal(got, want)
        ctx.tgrad_destroy()


def test_sparse_indices_all_equal_and_zero_tensors():
    for val in (0.0, 1.0 + 1.0j):
        g = np.full((9, 8, 7), val, dtype=np.complex64)
        ctx = make_gpu_ctx(T, g.shape, (1, 1, 1), 100, refresh_every=0)
        ctx.tgrad_refresh_factors(T.to_device_grad(g))
        assert np.array_equal(ctx.tgrad_get_state(T.STATE_INDICES), np.arange(100))


@pytest.mark.parametrize("shape,seed,dt", SEL_CASES)
def test_random_support_bit_exact(shape, seed, dt):
    """The rand-k rule: same counter-based keys on both sides, so the support is bit-exact; it
    depends on (seed, step count) and not on the gradient."""
    g = synth.small_case(shape, seed, dtype=dt)
    I = int(np.prod(shape))
    gd = T.to_device_grad(g)
    seeds = (0, seed, (seed << 40) | 12345, (1 << 64) - 1)
    for j, k in enumerate(sorted(set([0, 1, I // 100 + 1, I // 7, I // 2, I - 1, I]))):
        sd = seeds[j % len(seeds)]
        _announce("rand-k", shape, dt, "k=", k, "seed=", sd)
        ctx = make_gpu_ctx(T, shape, [1] * len(shape), k, grad_dtype=T.TGRAD_CBF16 if dt == "cbf16" else 0,
                           refresh_every=0, select_rule=T.TGRAD_SELECT_RANDOM, select_seed=sd)
        for t in (0, 7, (1 << 32) + 3):
            ctx.tgrad_set_state(T.STATE_STEP, np.array([t], dtype=np.int64))
            ctx.tgrad_refresh_factors(gd)
            got = ctx.tgrad_get_state(T.STATE_INDICES)
            assert np.array_equal(got, O.sparse_indices_random(I, k, sd, t))
        ctx.tgrad_destroy()


def test_random_rule_end_to_end():
    w = synth.WORKLOADS["cfg1"]
    _announce("cfg1 end to end, rand-k support")
    info, W0 = _end_to_end(w, 10, select_rule=T.TGRAD_SELECT_RANDOM, select_seed=2025)
    assert all(info["omega_equal"]) and len(info["omega_equal"]) == 2
    st = info["state"]
    assert np.array_equal(st.omega, O.sparse_indices_random(w.numel, w.k, 2025, (9 // w.T) * w.T))
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)


# ------------------------------------------------------------------ factors
@pytest.mark.parametrize("shape,ranks,k,seed", [
    ((16, 16, 8, 5), (8, 8, 4, 3), 103, 21),
    ((7, 5, 3, 2), (1, 1, 1, 1), 4, 22),
    ((33, 20, 9), (5, 20, 2), 60, 23),
    ((40, 130, 6), (10, 33, 6), 0, 24),
])
def test_gram_and_factors_match_oracle(shape, ranks, k, seed):
    _announce("factors", shape, ranks, k)
    g = synth.small_case(shape, seed, outlier_frac=(1, 100))
    ctx = make_gpu_ctx(T, shape, ranks, k, refresh_every=0)
    ctx.tgrad_refresh_factors(T.to_device_grad(g))
    om = O.sparse_indices(g, k)
    assert np.array_equal(ctx.tgrad_get_state(T.STATE_INDICES), om)
    X = O.remove_sparse(O.to_complex128(g), om)
    Uo = O.tucker_factors(X, ranks)
    for n in range(len(shape)):
        U = ctx.tgrad_get_state(T.STATE_FACTOR0 + n)
        if ranks[n] == shape[n]:
            assert np.array_equal(U, np.eye(shape[n], dtype=np.complex64))
            continue
        A = ctx.tgrad_get_state(T.STATE_GRAM0 + n)
        Ao = O.mode_gram(X, n)
        assert np.linalg.norm(A - Ao) <= 1e-12 * np.linalg.norm(Ao)
        assert np.max(np.abs(U.conj().T @ U - np.eye(ranks[n]))) < 1e-5          # orthonormal (fp32 storage)
        assert projector_distance(U, Uo[n]) < PROJ_TOL
        # individual eigenvectors, same phase convention (eigenvalues of random data are simple)
        assert np.max(np.abs(U - Uo[n])) < 1e-4


def test_exact_low_rank_gradient_gives_planted_subspace():
    rng = np.random.default_rng(31)
    shape, ranks = (24, 18, 10), (3, 4, 2)
    Q = [np.linalg.qr(rng.standard_normal((i, r)) + 1j * rng.standard_normal((i, r)))[0] for i, r in zip(shape, ranks)]
    core = rng.standard_normal(ranks) + 1j * rng.standard_normal(ranks)
    g = O.reconstruct(core, Q).astype(np.complex64)
    ctx = make_gpu_ctx(T, shape, ranks, 0, refresh_every=0)
    ctx.tgrad_refresh_factors(T.to_device_grad(g))
    for n in range(3):
        assert projector_distance(ctx.tgrad_get_state(T.STATE_FACTOR0 + n), Q[n]) < 1e-4


# ------------------------------------------------------------------ the three kernel tiers, small
FUSED_SHAPES = [
    ((16, 32, 32, 9), (4, 8, 8, 4), 300),          # one tile per slab
    ((16, 32, 64, 5), (4, 8, 16, 2), 200),         # two tiles per slab
    ((16, 32, 32, 33), (4, 8, 8, 8), 500),         # odd last extent, 9 pieces per lane and tile
    ((8, 64, 32, 35), (4, 8, 8, 6), 500),          # odd last extent, the long-row variant (17 pieces, 33 row pairs)
    ((16, 32, 32, 8), (4, 8, 8, 4), 300),          # even last extent: padded LDS rows
    ((16, 32, 32, 9), (4, 8, 8, 4), 45000),        # more than 64 support entries in every tile
]


@pytest.mark.parametrize("shape,ranks,k", FUSED_SHAPES)
def test_fused_tier_small_shapes(shape, ranks, k):
    """Shapes that take the fused kernels (modes N-1 and N in one pass) at a size the oracle runs
    whole; the launch counts prove which tier ran."""
    _announce("fused tier", shape, ranks, k)
    grads = [synth.small_case(shape, 500 + t, outlier_frac=(1, 200)) for t in range(6)]
    rng = np.random.default_rng(6)
    W0 = ((rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * 0.02).astype(np.complex64)
    info = run_both(T, shape, ranks, k, grads, W0, refresh_every=4, lr=2e-3, weight_decay=0.01)
    assert all(info["omega_equal"])
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)
    ctx = info["ctx"]
    ctx.tgrad_set_profiling(True)
    ctx.tgrad_step(T.to_device_weight(W0), T.to_device_grad(grads[0]))
    times = ctx.tgrad_get_kernel_times()
    # modes N and N-1 inside the first / last kernel, mode 1 (both ways) + AdamUpdate inside the core kernel
    assert times["core"]["launches"] == 1
    assert times["project"]["launches"] == len(shape) - 3 and times["backproject"]["launches"] == len(shape) - 3


CORE2_SHAPES = [
    ((128, 40, 32, 13), (8, 6, 32, 12), 4000, "us_lr"),      # second extent: one full tile + a ragged one
    ((128, 41, 32, 13), (32, 32, 32, 12), 4000, "us_lr"),    # odd second extent, full ranks in the two leading modes
    ((128, 128, 32, 13), (32, 32, 32, 12), 30000, "lr_us"),  # the headline's leading modes, low rank first
    ((128, 40, 32, 9), (8, 6, 16, 6), 2000, "us_lr"),        # 96 columns: one column per workgroup
    ((128, 33, 32, 9), (8, 6, 20, 5), 2000, "sum"),          # one column per workgroup, odd rank of the last mode
]


@pytest.mark.parametrize("shape,ranks,k,order", CORE2_SHAPES)
def test_two_mode_core_kernel_tier(shape, ranks, k, order):
    """Four-way tensors with a first extent of 128 and at least 192 column pairs (or, failing that, 96
    columns) behind the two leading modes: both leading modes (both ways) and AdamUpdate on the core
    run as ONE launch between the fused first projection and the fused update."""
    _announce("two-mode core kernel", shape, ranks, k)
    grads = [synth.small_case(shape, 900 + t, outlier_frac=(1, 200)) for t in range(5)]
    rng = np.random.default_rng(8)
    W0 = ((rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * 0.02).astype(np.complex64)
    info = run_both(T, shape, ranks, k, grads, W0, refresh_every=3, lr=2e-3, weight_decay=0.01,
                    order=getattr(T, "TGRAD_ORDER_" + order.upper()))
    assert all(info["omega_equal"])
    check_parity(info, W0)
    ctx = info["ctx"]
    ctx.tgrad_set_profiling(True)
    ctx.tgrad_step(T.to_device_weight(W0), T.to_device_grad(grads[0]))
    times = ctx.tgrad_get_kernel_times()
    assert times["core"]["launches"] == 1
    assert "project" not in times and "backproject" not in times          # kernels that never ran are not listed


# ------------------------------------------------------------------ weights stored as bf16 pairs
def _bf16_weights(shape, seed):
    rng = np.random.default_rng(seed)
    return O.complex_to_bf16_pairs((rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * 0.02)


BF16W_CASES = [
    # shape, ranks, k, gradient dtype            kernel tier
    ((16, 16, 8, 5), (8, 8, 4, 3), 103, "c64"),      # matrix-core, unfused
    ((16, 32, 32, 9), (4, 8, 8, 4), 300, "c64"),     # fused
    ((16, 32, 64, 5), (4, 8, 16, 2), 200, "cbf16"),  # fused, half-precision gradients too
    ((7, 5, 3), (3, 2, 2), 9, "c64"),                # last tile ragged: 3 rows x 3 elements
    ((9, 7, 6), (3, 3, 2), 11, "c64"),               # tail of 2 elements after the whole pieces
    ((8, 7, 40), (2, 2, 36), 30, "c64"),             # generic kernels (last-mode rank above 32)
    ((5, 4, 3, 1), (2, 2, 2, 1), 3, "c64"),          # generic kernels (last extent 1)
    ((128, 40, 32, 17), (8, 6, 32, 12), 4000, "c64"),  # fused + two-mode core kernel, last extent 17 (compile-time stage B)
]


@pytest.mark.parametrize("shape,ranks,k,dt", BF16W_CASES)
def test_bf16_weights_single_steps(shape, ranks, k, dt):
    """Each step starts from the oracle's bits: the GPU (float32 arithmetic) and the oracle
    (float64) may round differently only where the exact result sits within the float32 noise of
    a bf16 rounding boundary: at most one bf16 ulp apart (or, next to zero, 1e-3 * lr apart in
    value), on a small share of the entries."""
    _announce("bf16 weights, single steps", shape, ranks, k, dt)
    grads = [synth.small_case(shape, 600 + t, dtype=dt) for t in range(6)]
    info = run_both_bf16_weights(T, shape, ranks, k, grads, _bf16_weights(shape, 7), resync=True,
                                 grad_dtype=T.TGRAD_CBF16 if dt == "cbf16" else 0,
                                 refresh_every=4, lr=2e-3, weight_decay=0.01)
    I = int(np.prod(shape))
    for worst, frac in info["stats"]:
        assert worst <= 1
        assert frac <= max(5e-3, 2.0 / (2 * I))
    assert np.array_equal(info["ctx"].tgrad_get_state(T.STATE_INDICES), info["state"].omega)
    assert rel_err(info["ctx"].tgrad_get_state(T.STATE_SPARSE_M), info["state"].M_S) < 1e-5


def test_bf16_weights_ten_free_running_steps():
    w = synth.WORKLOADS["cfg1"]
    grads = [synth.gradient(w, t) for t in range(10)]
    W0 = _bf16_weights(w.shape, 8)
    info = run_both_bf16_weights(T, w.shape, w.ranks, w.k, grads, W0, refresh_every=w.T, lr=w.lr)
    worst, frac = info["stats"][-1]
    assert worst <= 2 and frac < 1e-2                      # single flips persist; they do not grow
    moved = np.count_nonzero(bf16_ordinal(info["W_gpu"]) != bf16_ordinal(W0))
    assert moved > 0.5 * 2 * w.numel                        # the update is visible at bf16 resolution
    a = O.bf16_pairs_to_complex(info["W_gpu"]) - O.bf16_pairs_to_complex(W0)
    b = O.bf16_pairs_to_complex(info["W_oracle"]) - O.bf16_pairs_to_complex(W0)
    assert np.linalg.norm(a - b) <= 1e-2 * np.linalg.norm(b)


# ------------------------------------------------------------------ composition orders
ORDER_CASES = [
    # shape, ranks, k, gradient dtype                 kernel tier
    ((16, 16, 8, 5), (8, 8, 4, 3), 103, "c64"),       # matrix-core, unfused
    ((16, 32, 32, 9), (4, 8, 8, 4), 300, "c64"),      # fused
    ((6, 5, 4, 3, 5), (2, 2, 2, 2, 2), 18, "cbf16"),  # five modes, half-precision gradients
    ((8, 7, 40), (2, 2, 36), 30, "c64"),              # generic last-mode kernels
    ((33, 20, 9), (5, 20, 2), 60, "c64"),             # one mode at full rank
]   # (no matrix here: stepping a matrix on its own refresh gradient makes the core exactly diagonal,
    #  see test_order2_tensor_with_explicit_refresh)


@pytest.mark.parametrize("order", ["lr_us", "sum"])
@pytest.mark.parametrize("shape,ranks,k,dt", ORDER_CASES)
def test_composition_orders_end_to_end(shape, ranks, k, dt, order):
    """Low rank first (the sparse part on the residual of the low-rank approximation) and the
    additive composition, against the oracle: support at every refresh, factors, weights."""
    _announce("order", order, shape, ranks, k, dt)
    oid = T.TGRAD_ORDER_LR_US if order == "lr_us" else T.TGRAD_ORDER_SUM
    grads = [synth.small_case(shape, 800 + t, dtype=dt) for t in range(7)]
    rng = np.random.default_rng(10)
    W0 = ((rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * 0.02).astype(np.complex64)
    info = run_both(T, shape, ranks, k, grads, W0, grad_dtype=T.TGRAD_CBF16 if dt == "cbf16" else 0,
                    refresh_every=3, lr=2e-3, lam=0.7, alpha=1.2, order=oid)
    assert all(info["omega_equal"]) and len(info["omega_equal"]) == 3
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)
    st, ctx = info["state"], info["ctx"]
    assert rel_err(ctx.tgrad_get_state(T.STATE_SPARSE_M), st.M_S) < 1e-4
    assert rel_err(ctx.tgrad_get_state(T.STATE_CORE_M), st.M_L) < 1e-4
    if order == "lr_us" and len(shape) > 2:
        # the support is that of the residual, not of the gradient itself
        assert not np.array_equal(st.omega, O.sparse_indices(grads[6], k))


def test_low_rank_first_with_hooi_and_random_support():
    w = synth.WORKLOADS["cfg1"]
    info, W0 = _end_to_end(w, 10, order=T.TGRAD_ORDER_LR_US, hooi_sweeps=1, select_rule=T.TGRAD_SELECT_RANDOM,
                           select_seed=77)
    assert all(info["omega_equal"]) and len(info["omega_equal"]) == 2
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)


# ------------------------------------------------------------------ HOOI sweeps, warm restart
def test_hooi_refresh_matches_oracle_cfg1():
    """Two refinement sweeps after HOSVD.  On this noise-like tensor the refined factors are far
    from the HOSVD ones (projector distance 0.2 ... 0.7), so agreement is not inherited from the
    HOSVD test."""
    w = synth.WORKLOADS["cfg1"]
    _announce("cfg1, 2 HOOI sweeps")
    info, W0 = _end_to_end(w, 10, hooi_sweeps=2)
    assert all(info["omega_equal"]) and len(info["omega_equal"]) == 2
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)
    g = synth.gradient(w, 5)                                       # the gradient of the last refresh
    X = O.remove_sparse(O.to_complex128(g), info["state"].omega)
    hosvd = O.tucker_factors(X, w.ranks)
    ctx = info["ctx"]
    far = [projector_distance(ctx.tgrad_get_state(T.STATE_FACTOR0 + n), hosvd[n]) for n in range(4)]
    assert min(far) > 0.05


def test_hooi_warm_restart_matches_oracle():
    w = synth.WORKLOADS["cfg1"]
    _announce("cfg1, 1 HOOI sweep, warm restart")
    info, W0 = _end_to_end(w, 12, hooi_sweeps=1, warm_restart=True)
    assert all(info["omega_equal"]) and len(info["omega_equal"]) == 3
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)
    # the restart matters: a cold start on the last refresh's gradient gives other factors
    g = synth.gradient(w, 10)
    X = O.remove_sparse(O.to_complex128(g), info["state"].omega)
    cold = O.tucker_factors(X, w.ranks, hooi_sweeps=1)
    ctx = info["ctx"]
    assert max(projector_distance(ctx.tgrad_get_state(T.STATE_FACTOR0 + n), cold[n]) for n in range(4)) > 10 * PROJ_TOL


def test_hooi_planted_low_rank_cfg2():
    w = synth.WORKLOADS["cfg2"]
    _announce("cfg2, 1 HOOI sweep")
    info, W0 = _end_to_end(w, 6, refresh_every=5, hooi_sweeps=1)
    assert all(info["omega_equal"]) and len(info["omega_equal"]) == 2
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)


@pytest.mark.parametrize("shape,ranks,k,dt,sweeps", [
    ((7, 5, 3, 2), (3, 2, 2, 1), 3, "c64", 2),
    ((6, 5, 4, 3, 5), (2, 2, 2, 2, 2), 18, "cbf16", 1),
    ((3, 4, 2, 3, 2, 5), (2, 2, 1, 2, 1, 3), 7, "c64", 1),
    ((33, 20, 9), (5, 20, 2), 60, "c64", 2),                        # one mode at full rank (identity factor)
    ((40, 9, 66), (6, 3, 9), 0, "c64", 1),                          # no sparse part, last-mode rank 9
])
def test_hooi_odd_shapes(shape, ranks, k, dt, sweeps):
    """Ranks obey r_n <= prod of the other ranks: beyond that the compressed unfolding is rank
    deficient and the trailing factor columns are arbitrary on both sides."""
    _announce("HOOI odd shape", shape, ranks, k, dt, sweeps)
    grads = [synth.small_case(shape, 300 + t, dtype=dt) for t in range(6)]
    rng = np.random.default_rng(5)
    W0 = ((rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * 0.02).astype(np.complex64)
    info = run_both(T, shape, ranks, k, grads, W0, grad_dtype=T.TGRAD_CBF16 if dt == "cbf16" else 0,
                    refresh_every=4, hooi_sweeps=sweeps, warm_restart=(sweeps == 1), lr=2e-3)
    assert all(info["omega_equal"])
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)


def test_hooi_order2_factors():
    """N = 2: compares the factors only (a step on the refresh gradient makes the core exactly
    diagonal and Adam amplifies the rounding noise of its vanishing entries)."""
    shape, ranks, k = (9, 6), (3, 3), 5
    g = synth.small_case(shape, 77)
    ctx = make_gpu_ctx(T, shape, ranks, k, refresh_every=0, hooi_sweeps=3)
    st = O.State(shape, O.Hyper(ranks=ranks, k=k, T=0, hooi_sweeps=3))
    ctx.tgrad_refresh_factors(T.to_device_grad(g))
    O.refresh(st, g)
    assert np.array_equal(ctx.tgrad_get_state(T.STATE_INDICES), st.omega)
    for n in range(2):
        assert projector_distance(ctx.tgrad_get_state(T.STATE_FACTOR0 + n), st.U[n]) < PROJ_TOL


# ------------------------------------------------------------------ step with injected state
def test_step_with_injected_support_and_factors():
    """Kernel arithmetic only: Omega and U come from the oracle, so eigen-sensitivity is out."""
    w = synth.WORKLOADS["cfg1"]
    g0 = synth.gradient(w, 0)
    st = O.State(w.shape, O.Hyper(ranks=w.ranks, k=w.k, T=0))
    O.refresh(st, g0)
    ctx = make_gpu_ctx(T, w.shape, w.ranks, w.k, refresh_every=0)
    W0 = synth.initial_weight(w)
    Wd = T.to_device_weight(W0)
    import ctypes
    rc = ctx.lib.tgrad_step(ctx.handle, Wd.data_ptr(), T.to_device_grad(g0).data_ptr())
    assert rc == T.TGRAD_ERR_NOT_READY
    ctx.tgrad_set_state(T.STATE_INDICES, st.omega)
    for n in range(4):
        ctx.tgrad_set_state(T.STATE_FACTOR0 + n, st.U[n])
    Wo = W0.astype(np.complex128)
    for t in range(10):
        g = synth.gradient(w, t)
        ctx.tgrad_step(Wd, T.to_device_grad(g))
        Wo = O.step(st, Wo, g)
        if t == 0:
            assert rel_err(ctx.tgrad_get_state(T.STATE_SPARSE_G), O.to_complex128(g).reshape(-1)[st.omega]) == 0.0
            Ro = O.compress(O.remove_sparse(O.to_complex128(g), st.omega), st.U)
            assert rel_err(ctx.tgrad_get_state(T.STATE_CORE_G), Ro) < 1e-5
    Wg = T.weight_to_host(Wd)
    assert ctx.t == 10
    check_parity({"W_gpu": Wg, "W_oracle": Wo, "ctx": ctx, "state": st, "lr": 1e-3, "steps": 10}, W0)
    assert rel_err(ctx.tgrad_get_state(T.STATE_CORE_M), st.M_L) < 1e-4
    assert rel_err(ctx.tgrad_get_state(T.STATE_SPARSE_V), st.V_S) < 1e-4


# ------------------------------------------------------------------ end to end
def _end_to_end(w, steps, scale=1.0, **over):
    grads = [synth.gradient(w, t, scale=scale) for t in range(steps)]
    W0 = synth.initial_weight(w)
    kw = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, alpha=w.alpha, lam=w.lam,
              weight_decay=w.weight_decay, refresh_every=w.T)
    kw.update(over)
    return run_both(T, w.shape, w.ranks, w.k, grads, W0,
                    grad_dtype=T.TGRAD_CBF16 if w.grad_dtype == "cbf16" else 0, **kw), W0


def test_cfg1_ten_steps_end_to_end():
    w = synth.WORKLOADS["cfg1"]
    _announce("cfg1 end to end")
    info, W0 = _end_to_end(w, 10)
    assert all(info["omega_equal"]) and len(info["omega_equal"]) == 2
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)


def test_cfg1_sixty_steps_no_drift():
    """Six times the protocol's length, twelve refreshes: the difference to the oracle stays at the
    float32 rounding level instead of growing with the step count."""
    w = synth.WORKLOADS["cfg1"]
    _announce("cfg1, 60 steps")
    info, W0 = _end_to_end(w, 60)
    assert all(info["omega_equal"]) and len(info["omega_equal"]) == 12
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)
    st, ctx = info["state"], info["ctx"]
    assert rel_err(ctx.tgrad_get_state(T.STATE_CORE_V), st.V_L) < 1e-4
    assert rel_err(ctx.tgrad_get_state(T.STATE_SPARSE_V), st.V_S) < 1e-4
    assert ctx.t == 60


def test_cfg1_rescaled_gradients():
    """Gradients of order 1e-4 (the paper notes moments of order 1e-5)."""
    w = synth.WORKLOADS["cfg1"]
    info, W0 = _end_to_end(w, 10, scale=1e-4)
    assert all(info["omega_equal"])
    check_parity(info, W0)


@pytest.mark.parametrize("shape,ranks,k,dt", [
    ((7, 5, 3, 2), (1, 1, 1, 1), 3, "c64"),
    ((7, 5, 3, 2), (3, 2, 2, 1), 0, "c64"),
    ((6, 5, 4, 3, 5), (2, 2, 2, 2, 2), 18, "cbf16"),
    ((3, 4, 2, 3, 2, 5), (2, 2, 1, 2, 1, 3), 7, "c64"),
    ((33, 20, 9), (5, 20, 2), 60, "c64"),
])
def test_odd_shapes_end_to_end(shape, ranks, k, dt):
    _announce("odd shape", shape, ranks, k, dt)
    grads = [synth.small_case(shape, 100 + t, dtype=dt) for t in range(10)]
    rng = np.random.default_rng(3)
    W0 = ((rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * 0.02).astype(np.complex64)
    info = run_both(T, shape, ranks, k, grads, W0, grad_dtype=T.TGRAD_CBF16 if dt == "cbf16" else 0,
                    refresh_every=4, alpha=0.8, lam=1.3, weight_decay=0.01, lr=2e-3)
    assert all(info["omega_equal"])
    assert max(max(d) for d in info["proj_dist"]) < PROJ_TOL
    check_parity(info, W0)


def test_order2_tensor_with_explicit_refresh():
    """N = 2 (the matrix case).  Factors come from an explicit refresh on a DIFFERENT gradient:
    refreshing on the gradient that is then stepped makes the compressed gradient exactly
    diagonal (it is the SVD), and Adam's M / (sqrt(V) + eps) turns the rounding noise of the
    vanishing off-diagonal entries into O(1) values in any finite precision."""
    shape, ranks, k = (9, 6), (4, 3), 5
    _announce("order-2", shape, ranks, k)
    ctx = make_gpu_ctx(T, shape, ranks, k, refresh_every=0, lr=2e-3)
    st = O.State(shape, O.Hyper(ranks=ranks, k=k, T=0, lr=2e-3))
    g_ref = synth.small_case(shape, 77)
    ctx.tgrad_refresh_factors(T.to_device_grad(g_ref))
    O.refresh(st, g_ref)
    assert np.array_equal(ctx.tgrad_get_state(T.STATE_INDICES), st.omega)
    W0 = synth.small_case(shape, 998) * np.float32(0.02)
    Wd = T.to_device_weight(W0)
    Wo = W0.astype(np.complex128)
    for t in range(10):
        g = synth.small_case(shape, 300 + t)
        ctx.tgrad_step(Wd, T.to_device_grad(g))
        Wo = O.step(st, Wo, g)
    Wg = T.weight_to_host(Wd)
    check_parity({"W_gpu": Wg, "W_oracle": Wo, "ctx": ctx, "state": st, "lr": 2e-3, "steps": 10}, W0)


@pytest.mark.parametrize("mode", ["all_sparse", "full_rank"])
def test_degenerate_cases_are_dense_adam(mode):
    shape = (6, 5, 4)
    I = 120
    ranks, k = ((2, 1, 3), I) if mode == "all_sparse" else (shape, 0)
    grads = [synth.small_case(shape, 200 + t) for t in range(10)]
    W0 = synth.small_case(shape, 999) * np.float32(0.02)
    info = run_both(T, shape, ranks, k, grads, W0, refresh_every=3, weight_decay=0.1, lr=1e-2)
    Wd = W0.astype(np.complex128)
    M = np.zeros(shape, complex)
    V = np.zeros(shape)
    f32 = lambda x: float(np.float32(x))                   # the values the ABI carries
    for t, g in enumerate(grads):
        Wd, M, V = O.dense_complex_adam_step(Wd, g, M, V, t, f32(1e-2), f32(0.9), f32(0.999), f32(1e-8), f32(0.1))
    assert rel_err(info["W_oracle"], Wd) < 1e-14
    assert rel_err(info["W_gpu"], Wd) < 2e-6
    assert rel_err(info["W_gpu"] - W0, Wd - W0) < 1e-5


def test_two_runs_are_bit_identical():
    w = synth.WORKLOADS["cfg1"]
    outs = []
    for _ in range(2):
        ctx = make_gpu_ctx(T, w.shape, w.ranks, w.k, refresh_every=w.T)
        Wd = T.to_device_weight(synth.initial_weight(w))
        for t in range(6):
            ctx.tgrad_step(Wd, T.to_device_grad(synth.gradient(w, t)))
        outs.append((T.weight_to_host(Wd), ctx.tgrad_get_state(T.STATE_CORE_M), ctx.tgrad_get_state(T.STATE_FACTOR0)))
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_checkpoint_restore_is_bit_identical():
    w = synth.WORKLOADS["cfg1"]
    grads = [synth.gradient(w, t) for t in range(8)]
    ctx = make_gpu_ctx(T, w.shape, w.ranks, w.k, refresh_every=w.T)
    Wd = T.to_device_weight(synth.initial_weight(w))
    for t in range(4):
        ctx.tgrad_step(Wd, T.to_device_grad(grads[t]))
    items = [T.STATE_STEP, T.STATE_INDICES, T.STATE_CORE_M, T.STATE_CORE_V, T.STATE_SPARSE_M, T.STATE_SPARSE_V] + \
            [T.STATE_FACTOR0 + n for n in range(4)]
    saved = {it: ctx.tgrad_get_state(it) for it in items}
    W_saved = T.weight_to_host(Wd).copy()
    for t in range(4, 8):
        ctx.tgrad_step(Wd, T.to_device_grad(grads[t]))
    W_a = T.weight_to_host(Wd)
    ctx2 = make_gpu_ctx(T, w.shape, w.ranks, w.k, refresh_every=w.T)
    for it in items:
        ctx2.tgrad_set_state(it, saved[it])
    Wd2 = T.to_device_weight(W_saved)
    for t in range(4, 8):
        ctx2.tgrad_step(Wd2, T.to_device_grad(grads[t]))
    assert ctx2.t == 8
    assert np.array_equal(T.weight_to_host(Wd2), W_a)


@pytest.mark.parametrize("case", [FUSED_SHAPES[1], CORE2_SHAPES[0][:3]])
def test_checkpoint_restore_fused_tier(case):
    """The same on shapes that take the fused kernels (and the two-mode core kernel): their factor
    copies and operand tables must follow tgrad_set_state (they are rebuilt when a factor is written,
    not on every step)."""
    shape, ranks, k = case
    grads = [synth.small_case(shape, 700 + t) for t in range(6)]
    rng = np.random.default_rng(9)
    W0 = ((rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * 0.02).astype(np.complex64)
    ctx = make_gpu_ctx(T, shape, ranks, k, refresh_every=4)
    Wd = T.to_device_weight(W0)
    for t in range(3):
        ctx.tgrad_step(Wd, T.to_device_grad(grads[t]))
    items = [T.STATE_STEP, T.STATE_INDICES, T.STATE_CORE_M, T.STATE_CORE_V, T.STATE_SPARSE_M, T.STATE_SPARSE_V] + \
            [T.STATE_FACTOR0 + n for n in range(4)]
    saved = {it: ctx.tgrad_get_state(it) for it in items}
    W_saved = T.weight_to_host(Wd).copy()
    ctx.tgrad_step(Wd, T.to_device_grad(grads[3]))          # t = 3: no refresh, uses the restored factors
    W_a = T.weight_to_host(Wd)
    ctx2 = make_gpu_ctx(T, shape, ranks, k, refresh_every=4)
    for it in items:
        ctx2.tgrad_set_state(it, saved[it])
    Wd2 = T.to_device_weight(W_saved)
    ctx2.tgrad_step(Wd2, T.to_device_grad(grads[3]))
    assert np.array_equal(T.weight_to_host(Wd2), W_a)


def test_set_state_rejects_bad_indices():
    ctx = make_gpu_ctx(T, (6, 5, 4), (2, 2, 2), 3, refresh_every=0)
    for bad in ([0, 0, 1], [2, 1, 3], [0, 1, 120], [-1, 0, 1]):
        with pytest.raises(T.TgradError):
            ctx.tgrad_set_state(T.STATE_INDICES, np.array(bad, dtype=np.int64))
    with pytest.raises(T.TgradError):
        ctx.tgrad_set_state(T.STATE_SPARSE_G, np.zeros(3, np.complex64))     # read-only item


# ------------------------------------------------------------------ failure detection
def test_eigen_solve_reports_convergence_and_a_forced_sweep_limit():
    """Every compressed mode's solve reports (stalled, Jacobi sweeps, declined).  By default the
    tridiagonal solver delivers the factor (no Jacobi sweep); asked for by its sweep budget, the
    Jacobi solver ends by itself within the budget and gives the same factors; with a budget of
    one sweep (forced from the host) it stops with rotations left: the factor is still delivered
    and tgrad_get_state says NOT_CONVERGED."""
    shape, ranks, k = (24, 18, 10), (5, 4, 3), 20
    g = synth.small_case(shape, 905)
    ctx = make_gpu_ctx(T, shape, ranks, k, refresh_every=0)
    ctx.tgrad_refresh_factors(T.to_device_grad(g))
    fast = []
    for n in range(3):
        stalled, sweeps, declined = ctx.tgrad_get_state(T.STATE_EIG_INFO0 + n)
        assert (stalled, sweeps, declined) == (0, 0, 0)
        fast.append(ctx.tgrad_get_state(T.STATE_FACTOR0 + n))
    ctx.tgrad_destroy()
    ctx = make_gpu_ctx(T, shape, ranks, k, refresh_every=0, eig_max_sweeps=30)
    ctx.tgrad_refresh_factors(T.to_device_grad(g))
    for n in range(3):
        stalled, sweeps, declined = ctx.tgrad_get_state(T.STATE_EIG_INFO0 + n)
        assert stalled == 0 and 2 <= sweeps <= 30
        U = ctx.tgrad_get_state(T.STATE_FACTOR0 + n)
        assert np.max(np.abs(U - fast[n])) < 1e-6                      # two solvers, one answer
    ctx.tgrad_destroy()
    ctx = make_gpu_ctx(T, shape, ranks, k, refresh_every=0, eig_max_sweeps=1)
    ctx.tgrad_refresh_factors(T.to_device_grad(g))
    for n in range(3):
        stalled, sweeps, declined = ctx.tgrad_get_state(T.STATE_EIG_INFO0 + n)
        assert stalled == 1 and sweeps == 1
        U = np.zeros((shape[n], ranks[n]), dtype=np.complex64)
        rc = ctx.lib.tgrad_get_state(ctx.handle, T.STATE_FACTOR0 + n, U.ctypes.data, U.nbytes)
        assert rc == T.TGRAD_ERR_NOT_CONVERGED
        assert np.all(np.isfinite(U.view(np.float32))) and np.linalg.norm(U) > 0   # delivered all the same
    # an injected factor is nobody's failed solve
    ctx.tgrad_set_state(T.STATE_FACTOR0, np.eye(shape[0], ranks[0], dtype=np.complex64))
    ctx.tgrad_destroy()


def test_eigen_solve_on_degenerate_clusters():
    """A gradient whose mode Gram matrices have exactly repeated eigenvalues (multiplicities 4, 2, 2
    and a simple tail) up to a perturbation at rounding level.  Any basis of a cluster is correct, so
    the check is what is unique: the solve ends by itself, the factor is orthonormal, and the energy
    it captures equals the sum of the leading eigenvalues (the rank does not cut a cluster)."""
    rng = np.random.default_rng(77)
    shape = (12, 12)
    sv = np.array([5, 5, 5, 5, 3, 3, 2, 2, 1, 0.5, 0.25, 0.125])
    Q1 = np.linalg.qr(rng.standard_normal((12, 12)) + 1j * rng.standard_normal((12, 12)))[0]
    Q2 = np.linalg.qr(rng.standard_normal((12, 12)) + 1j * rng.standard_normal((12, 12)))[0]
    g = ((Q1 * sv) @ Q2.conj().T).astype(np.complex64)
    for r in (4, 6, 8):
        ctx = make_gpu_ctx(T, shape, (r, r), 0, refresh_every=0)
        ctx.tgrad_refresh_factors(T.to_device_grad(g))
        X = O.to_complex128(g)
        for n in range(2):
            stalled, sweeps, declined = ctx.tgrad_get_state(T.STATE_EIG_INFO0 + n)
            assert stalled == 0 and sweeps <= 30
            assert declined in (0, 1)       # the clusters are split at float32 rounding level: either solver may take it
            U = ctx.tgrad_get_state(T.STATE_FACTOR0 + n).astype(np.complex128)
            assert np.max(np.abs(U.conj().T @ U - np.eye(r))) < 1e-5
            Xn = X if n == 0 else X.T
            captured = np.linalg.norm(U.conj().T @ Xn) ** 2
            assert abs(captured - np.sum(sv[:r] ** 2)) <= 1e-5 * np.sum(sv ** 2)
        ctx.tgrad_destroy()


def _matrix_with_singular_values(n, sv, seed):
    rng = np.random.default_rng(seed)
    Q1 = np.linalg.qr(rng.standard_normal((n, n)) + 1j * rng.standard_normal((n, n)))[0]
    Q2 = np.linalg.qr(rng.standard_normal((n, n)) + 1j * rng.standard_normal((n, n)))[0]
    return ((Q1 * sv) @ Q2.conj().T).astype(np.complex64)


@pytest.mark.parametrize("n", [2, 3, 5, 16, 17, 31, 33, 64, 65, 96, 127, 128])
def test_eigen_solve_over_extents_ranks_and_spectra(n):
    """The solver for extents up to 128 against the oracle's factors, column by column, on square
    matrices with prescribed singular values: a geometric decay over two decades (Gram eigenvalues
    over four: their smallest gap is still 5e-6 of the spectral radius at n = 128), a flat noise-like spectrum with gaps of 1e-3, and a pair of leading singular values
    1e-4 apart (a Gram gap of 2e-4 of the spectral radius: far above the threshold at which the
    tridiagonal path declines, small enough to stress inverse iteration).  Ranks 1, n / 4 and n - 1."""
    _announce("eigen-solve sweep", n)
    spectra = {
        "geometric": 10.0 ** (-2.0 * np.arange(n) / max(1, n - 1)),
        "flat": 1.0 - 1e-3 * np.arange(n),
        "close pair": np.concatenate(([1.0, 1.0 - 1e-4], 0.9 - 0.5 * np.arange(max(0, n - 2)) / max(1, n))),
    }
    for name, sv in spectra.items():
        g = _matrix_with_singular_values(n, sv[:n], 100 + n)
        X = O.to_complex128(g)
        for r in sorted({1, max(1, n // 4), n - 1}):
            ctx = make_gpu_ctx(T, (n, n), (r, r), 0, refresh_every=0)
            ctx.tgrad_refresh_factors(T.to_device_grad(g))
            Uo = O.tucker_factors(X, (r, r))
            for mode in range(2):
                stalled, sweeps, declined = ctx.tgrad_get_state(T.STATE_EIG_INFO0 + mode)
                assert (stalled, declined) == (0, 0), (name, r, mode)
                U = ctx.tgrad_get_state(T.STATE_FACTOR0 + mode).astype(np.complex128)
                assert np.max(np.abs(U.conj().T @ U - np.eye(r))) < 1e-5, (name, r, mode)
                assert projector_distance(U, Uo[mode]) < PROJ_TOL, (name, r, mode)
                # (both sides see the same float32 matrix and accumulate its Gram in float64: the pair's gap
                # divides errors of 1e-16, not of 1e-7)
                assert np.max(np.abs(U - Uo[mode])) < 1e-4, (name, r, mode)
            ctx.tgrad_destroy()


def test_exactly_repeated_eigenvalues_go_to_the_jacobi_solver():
    """A diagonal gradient with repeated entries: the Gram matrices are exactly diagonal with exactly
    repeated eigenvalues.  Inverse iteration cannot separate those, so the tridiagonal solver must
    decline and the Jacobi solver deliver: unit vectors, ordered by (eigenvalue descending, index
    ascending)."""
    sv = np.array([5, 5, 5, 5, 3, 3, 2, 2, 1, 0.5, 0.25, 0.125], dtype=np.float32)
    g = np.diag(sv).astype(np.complex64)
    for r in (3, 4, 7):
        ctx = make_gpu_ctx(T, (12, 12), (r, r), 0, refresh_every=0)
        ctx.tgrad_refresh_factors(T.to_device_grad(g))
        for n in range(2):
            stalled, sweeps, declined = ctx.tgrad_get_state(T.STATE_EIG_INFO0 + n)
            assert (stalled, declined) == (0, 1) and sweeps >= 1
            U = ctx.tgrad_get_state(T.STATE_FACTOR0 + n)
            assert np.array_equal(U, np.eye(12, r, dtype=np.complex64))
        ctx.tgrad_destroy()
    # and a zero gradient: nothing to separate at all
    ctx = make_gpu_ctx(T, (12, 12), (3, 3), 0, refresh_every=0)
    ctx.tgrad_refresh_factors(T.to_device_grad(np.zeros((12, 12), dtype=np.complex64)))
    assert tuple(ctx.tgrad_get_state(T.STATE_EIG_INFO0))[2] == 1
    assert np.array_equal(ctx.tgrad_get_state(T.STATE_FACTOR0), np.eye(12, 3, dtype=np.complex64))
    ctx.tgrad_destroy()


def test_calibration_probes_run_and_report_their_work():
    import torch
    sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    for kind, per_instr in ((0, 4096.0), (1, 2048.0)):
        fl = T.tgrad_calibration_mfma(kind, 100, sink)
        torch.cuda.synchronize()
        # 100 iterations round up to 128 (whole unrolled trips); 4 instructions each, 8 wavefronts per compute unit
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        assert fl == cus * 8 * 128 * 4 * per_instr
    assert float(sink.abs().sum()) == 0.0
    src = torch.arange(1 << 16, dtype=torch.int32, device="cuda:0")
    dst = torch.zeros_like(src)
    T.tgrad_calibration_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    # the tile stream rewrites its buffer with itself: 17 tiles of 1040 pieces in slabs of 4 -> 16 tiles move
    buf = torch.arange(17 * 1040 * 4 + 5, dtype=torch.int32, device="cuda:0")
    keep = buf.clone()
    assert T.tgrad_calibration_tile_stream(buf, 1040 * 16, 4) == 16 * 1040 * 16
    torch.cuda.synchronize()
    assert torch.equal(buf, keep)


def test_check_counts_non_finite_gradient_entries():
    shape, ranks, k = (16, 16, 8, 5), (8, 8, 4, 3), 103
    g = synth.small_case(shape, 31).copy()
    ctx = make_gpu_ctx(T, shape, ranks, k, refresh_every=0)
    import ctypes
    n = ctypes.c_int64(0)
    assert ctx.lib.tgrad_check(ctx.handle, ctypes.byref(n)) == T.TGRAD_ERR_NOT_READY
    ctx.tgrad_refresh_factors(T.to_device_grad(g))
    assert ctx.tgrad_check() == 0
    flat = g.reshape(-1)
    flat[5] = complex(np.inf, 0.0)
    flat[77] = complex(0.0, np.nan)
    flat[1234] = complex(3e19, 3e19)                       # finite parts, |g|^2 overflows float32
    ctx.tgrad_refresh_factors(T.to_device_grad(g))
    assert ctx.tgrad_check() == 3
    ctx.tgrad_destroy()
    ctx = make_gpu_ctx(T, shape, ranks, k, refresh_every=0, select_rule=T.TGRAD_SELECT_RANDOM)
    ctx.tgrad_refresh_factors(T.to_device_grad(g))
    assert ctx.lib.tgrad_check(ctx.handle, ctypes.byref(n)) == T.TGRAD_ERR_UNSUPPORTED
