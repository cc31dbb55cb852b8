"""Shared drivers for the GPU parity tests: run the same seeded job through the HIP library
(via its C ABI binding) and through the CPU oracle."""
from __future__ import annotations

import numpy as np

from oracle import tgrad_oracle as O


def projector_distance(Ua: np.ndarray, Ub: np.ndarray) -> float:
    """|| Ua Ua^H - Ub Ub^H ||_F / sqrt(r)"""
    Ua = np.asarray(Ua, dtype=np.complex128)
    Ub = np.asarray(Ub, dtype=np.complex128)
    r = Ua.shape[1]
    return float(np.linalg.norm(Ua @ Ua.conj().T - Ub @ Ub.conj().T) / np.sqrt(max(r, 1)))


def rel_err(a: np.ndarray, b: np.ndarray) -> float:
    den = float(np.linalg.norm(b))
    return float(np.linalg.norm(np.asarray(a, dtype=np.complex128) - b) / (den if den > 0 else 1.0))


def max_abs_err(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.max(np.abs(np.asarray(a, dtype=np.complex128) - b))) if np.size(b) else 0.0


# Element-wise bar on the update.  One step moves an entry by lr * |D| with |D| of order one (Adam's
# normalised direction), so an entry that is wrong in kind - a mis-scattered sparse value, a tile
# column from the wrong slab, a missed decay - is off by about lr; float32 arithmetic against the
# float64 oracle leaves about 1e-6 * lr per step.  1e-2 * lr * sqrt(steps) separates the two by
# orders of magnitude on both sides.
ENTRY_TOL = 1e-2
W_TOL = 1e-4          # || W_g - W_o ||_F / || W_o ||_F   (the stated bar)
DW_TOL = 1e-4         # the same on W_t - W_0: sensitive to the optimizer and not to W_0


def check_parity(info, W0, moments=True):
    """Weights as tensors (Frobenius, on W and on W - W0) AND entry by entry; Adam moments entry by
    entry relative to their largest entry."""
    Wg = np.asarray(info["W_gpu"], dtype=np.complex128)
    Wo = info["W_oracle"]
    lr, steps = info["lr"], info["steps"]
    assert np.all(np.isfinite(Wg.view(np.float64)))
    assert rel_err(Wg, Wo) < W_TOL
    dg, do = Wg - W0, Wo - W0
    assert rel_err(dg, do) < DW_TOL, rel_err(dg, do)
    worst = max_abs_err(dg, do)
    assert worst <= ENTRY_TOL * lr * max(1.0, np.sqrt(steps)), worst
    if moments:
        from paper_2501_02379_amd import tgrad as T
        ctx, st = info["ctx"], info["state"]
        for what, ref in ((T.STATE_CORE_M, st.M_L), (T.STATE_CORE_V, st.V_L),
                          (T.STATE_SPARSE_M, st.M_S), (T.STATE_SPARSE_V, st.V_S)):
            if ref.size == 0:
                continue
            got = ctx.tgrad_get_state(what).astype(ref.dtype)
            scale = float(np.max(np.abs(ref)))
            assert max_abs_err(got, ref) <= 1e-4 * scale + 1e-30, (what, max_abs_err(got, ref), scale)


def oracle_hyper(shape, ranks, k, **kw) -> O.Hyper:
    """The oracle's hyper-parameters for a library configuration.  The ABI carries lr, the decay
    rates, eps, alpha, lambda and the weight decay as float32, so the oracle is given exactly those
    values (as float64 numbers): both sides then solve the same problem."""
    def f32(name, default):
        return float(np.float32(kw.get(name, default)))
    return O.Hyper(ranks=tuple(ranks), k=int(k), lr=f32("lr", 1e-3), beta1=f32("beta1", 0.9),
                   beta2=f32("beta2", 0.999), eps=f32("eps", 1e-8), alpha=f32("alpha", 1.0),
                   lam=f32("lam", 1.0), weight_decay=f32("weight_decay", 0.0),
                   T=kw.get("refresh_every", 1), hooi_sweeps=kw.get("hooi_sweeps", 0),
                   warm_restart=bool(kw.get("warm_restart", False)),
                   order={0: "us_lr", 1: "lr_us", 2: "sum"}[kw.get("order", 0)],
                   select_rule="randk" if kw.get("select_rule", 0) == 1 else "topk",
                   select_seed=kw.get("select_seed", 0))


def make_gpu_ctx(T, shape, ranks, k, grad_dtype=0, **kw):
    cfg = T.make_config(shape, ranks, k, grad_dtype=grad_dtype, **kw)
    return T.Context(cfg)


def run_both(T, shape, ranks, k, grads, W0, grad_dtype=0, check_every_refresh=True, **kw):
    """Runs len(grads) steps on both sides.  Returns dict with final weights and per-refresh
    index/factor comparisons."""
    import torch
    ctx = make_gpu_ctx(T, shape, ranks, k, grad_dtype=grad_dtype, **kw)
    st = O.State(tuple(shape), oracle_hyper(shape, ranks, k, **kw))
    Wd = T.to_device_weight(W0)
    Wo = W0.astype(np.complex128)
    Tper = kw.get("refresh_every", 1)
    info = {"omega_equal": [], "proj_dist": [], "lr": kw.get("lr", 1e-3), "steps": 0}
    for t, g in enumerate(grads):
        info["steps"] = t + 1
        gd = T.to_device_grad(g)
        ctx.tgrad_step(Wd, gd)
        Wo = O.step(st, Wo, g)
        if check_every_refresh and Tper > 0 and t % Tper == 0:
            om = ctx.tgrad_get_state(T.STATE_INDICES)
            info["omega_equal"].append(bool(np.array_equal(om, st.omega)))
            info["proj_dist"].append([projector_distance(ctx.tgrad_get_state(T.STATE_FACTOR0 + n), st.U[n])
                                      for n in range(len(shape))])
    torch.cuda.synchronize()
    info["W_gpu"] = T.weight_to_host(Wd)
    info["W_oracle"] = Wo
    info["ctx"] = ctx
    info["state"] = st
    return info


def bf16_ordinal(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> integers that increase with the value (consecutive bf16 numbers differ by 1)."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.int32)
    mag = b & 0x7FFF
    return np.where(b & 0x8000, -mag, mag)


def run_both_bf16_weights(T, shape, ranks, k, grads, W0_bits, grad_dtype=0, resync=False, **kw):
    """Like run_both, with weights stored as bf16 pairs on both sides.  `resync`: before every step
    the GPU receives the oracle's current weights, so each step starts from identical bits and the
    comparison isolates one step's rounding.

    Per step it records (worst, frac): `frac` = share of the stored numbers whose bits differ;
    `worst` = largest difference in bf16 ulps among those that also differ by more than
    1e-3 * lr in value.  (Close to zero a bf16 ulp is far smaller than the float32 rounding noise
    of the update itself, about 1e-5 * lr, so there the distance in value is the meaningful one.)"""
    import torch
    ctx = make_gpu_ctx(T, shape, ranks, k, grad_dtype=grad_dtype, weight_dtype=T.TGRAD_CBF16, **kw)
    st = O.State(tuple(shape), oracle_hyper(shape, ranks, k, **kw))
    atol = 1e-3 * kw.get("lr", 1e-3)
    Wo = np.array(W0_bits, dtype=np.uint16, copy=True)
    Wd = T.to_device_weight(Wo)
    stats = []
    for g in grads:
        if resync:
            Wd = T.to_device_weight(Wo)
        ctx.tgrad_step(Wd, T.to_device_grad(g))
        Wo = O.step(st, Wo, g)
        torch.cuda.synchronize()
        Wg = T.weight_to_host(Wd)
        d = np.abs(bf16_ordinal(Wg) - bf16_ordinal(Wo))
        vg = (Wg.astype(np.uint32) << np.uint32(16)).view(np.float32)
        vo = (Wo.astype(np.uint32) << np.uint32(16)).view(np.float32)
        far = np.abs(vg.astype(np.float64) - vo.astype(np.float64)) > atol
        stats.append((int(d[far].max()) if far.any() else 0, float(np.count_nonzero(d)) / d.size))
    return {"stats": stats, "W_gpu": T.weight_to_host(Wd), "W_oracle": Wo, "ctx": ctx, "state": st}
