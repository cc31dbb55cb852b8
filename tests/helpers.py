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


def oracle_hyper(shape, ranks, k, **kw) -> O.Hyper:
    return O.Hyper(ranks=tuple(ranks), k=int(k), lr=kw.get("lr", 1e-3), beta1=kw.get("beta1", 0.9),
                   beta2=kw.get("beta2", 0.999), eps=kw.get("eps", 1e-8), alpha=kw.get("alpha", 1.0),
                   lam=kw.get("lam", 1.0), weight_decay=kw.get("weight_decay", 0.0),
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
    info = {"omega_equal": [], "proj_dist": []}
    for t, g in enumerate(grads):
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
