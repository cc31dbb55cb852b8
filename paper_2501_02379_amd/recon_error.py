"""Reconstruction-error diagnostic of the robust decomposition (a tool beside the hot path).

Section "Optimizer update" compares, on one complex 64^3 x 32 gradient of an FNO layer, the
distribution of |G - G~| for three one-shot approximations G~ of equal budget:
  (1) unstructured sparse 5 % first, then Tucker low rank 20 % on the rest   (Algorithm 1's order),
  (2) Tucker low rank 20 % first, then sparse 5 % of its residual,
  (3) pure Tucker low rank 25 %.
Here the decompositions are the LIBRARY's: one `tgrad_step` per strategy on the GPU leaves the
support Omega, the gathered sparse values, the compressed gradient (Tucker core) and the factors
in the context; this module only reads them back and rebuilds
    G~ = core x_1 U1 ... x_N UN  +  scatter(sparse values at Omega)
on the host to take the error statistics and a log-spaced histogram.  Nothing here is on the
optimizer's step path.

    python -m paper_2501_02379_amd.recon_error --out FILE
"""
from __future__ import annotations

import argparse
import sys
from typing import Dict, Sequence

import numpy as np

STRATEGIES = ("sparse 5% then low rank 20%", "low rank 20% then sparse 5%", "pure low rank 25%")


def _expand(core: np.ndarray, factors: Sequence[np.ndarray]) -> np.ndarray:
    """core x_1 U1 ... x_N UN on the host (float64 accumulation of the library's float32 values)."""
    D = np.asarray(core, dtype=np.complex128)
    for n, U in enumerate(factors):
        D = np.moveaxis(np.tensordot(np.asarray(U, dtype=np.complex128), D, axes=(1, n)), 0, n)
    return np.ascontiguousarray(D)


def library_approximation(g: np.ndarray, ranks: Sequence[int], k: int, order: int, device="cuda:0") -> Dict:
    """One refresh + step of the library on `g`; returns the pieces of its decomposition and the
    approximation G~ rebuilt from them."""
    import torch
    from . import tgrad as T
    cfg = T.make_config(g.shape, ranks, k, refresh_every=1, order=order, lr=1e-3)
    ctx = T.Context(cfg, device=device)
    W = torch.zeros(g.shape + (2,), dtype=torch.float32, device=device)
    ctx.tgrad_step(W, T.to_device_grad(g, device))
    torch.cuda.synchronize()
    out = {
        "omega": ctx.tgrad_get_state(T.STATE_INDICES),
        "sparse": ctx.tgrad_get_state(T.STATE_SPARSE_G),
        "core": ctx.tgrad_get_state(T.STATE_CORE_G),
        "factors": [ctx.tgrad_get_state(T.STATE_FACTOR0 + n) for n in range(len(g.shape))],
    }
    ctx.tgrad_destroy()
    approx = _expand(out["core"], out["factors"])
    if k > 0:
        approx.reshape(-1)[out["omega"]] += out["sparse"].astype(np.complex128)
    out["approx"] = approx
    return out


def error_statistics(err: np.ndarray) -> Dict[str, float]:
    e = np.asarray(err, dtype=np.float64).reshape(-1)
    return {"max": float(e.max()), "q999": float(np.quantile(e, 0.999)), "q99": float(np.quantile(e, 0.99)),
            "median": float(np.median(e)), "mean": float(e.mean()), "rms": float(np.sqrt(np.mean(e * e)))}


def histogram_edges(lo: float = 1e-3, hi: float = 1e4, per_decade: int = 4) -> np.ndarray:
    n = int(round(np.log10(hi / lo) * per_decade))
    return lo * 10.0 ** (np.arange(n + 1) / per_decade)


def run(g: np.ndarray, ranks20: Sequence[int], ranks25: Sequence[int], k5: int, device="cuda:0"):
    """|G - G~| of the three strategies, from the library's decompositions."""
    from . import tgrad as T
    X = g.astype(np.complex128)
    errs = []
    for ranks, k, order in ((ranks20, k5, T.TGRAD_ORDER_US_LR), (ranks20, k5, T.TGRAD_ORDER_LR_US),
                            (ranks25, 0, T.TGRAD_ORDER_US_LR)):
        parts = library_approximation(g, ranks, k, order, device)
        errs.append(np.abs(X - parts["approx"]))
    return errs


def report(errs, shape, ranks20, ranks25, k5) -> str:
    edges = histogram_edges()
    lines = [
        "Reconstruction error |G - G~| of three one-shot approximations of equal budget, from the library's",
        "own decompositions (support, sparse values, Tucker core and factors read back after one tgrad_step).",
        "Gradient: synthetic %s complex64 (planted low-rank signal + noise + Student-t outliers at 1 %% of the"
        % "x".join(map(str, shape)),
        "positions), stand-in for the FNO-layer gradient of the paper's reconstruction-error figure.",
        "ranks 20 %% = %s, ranks 25 %% = %s, k (5 %%) = %d" % (tuple(ranks20), tuple(ranks25), k5),
        "",
        "%-30s %12s %12s %12s %12s %12s" % ("strategy", "max", "q99.9", "q99", "mean", "rms"),
    ]
    for name, e in zip(STRATEGIES, errs):
        s = error_statistics(e)
        lines.append("%-30s %12.5g %12.5g %12.5g %12.5g %12.5g" % (name, s["max"], s["q999"], s["q99"], s["mean"], s["rms"]))
    lines += ["", "histogram (entries per bin of |G - G~|; first column: everything below %.0e)" % edges[0],
              "%-22s %14s %14s %14s" % ("bin", "sparse->lowrank", "lowrank->sparse", "lowrank only")]
    counts = []
    for e in errs:
        flat = e.reshape(-1)
        c, _ = np.histogram(flat, bins=edges)
        counts.append((int(np.count_nonzero(flat < edges[0])), c, int(np.count_nonzero(flat >= edges[-1]))))
    lines.append("%-22s %14d %14d %14d" % ("< %.3g" % edges[0], counts[0][0], counts[1][0], counts[2][0]))
    for b in range(len(edges) - 1):
        lines.append("%-22s %14d %14d %14d" % ("[%.3g, %.3g)" % (edges[b], edges[b + 1]), counts[0][1][b],
                                              counts[1][1][b], counts[2][1][b]))
    lines.append("%-22s %14d %14d %14d" % (">= %.3g" % edges[-1], counts[0][2], counts[1][2], counts[2][2]))
    return "\n".join(lines) + "\n"


def main(argv=None) -> int:
    from . import synth
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--out", default="-", help="text file to write (default: stdout)")
    args = ap.parse_args(argv)
    w = synth.RECON_DIAGNOSTIC
    ranks25 = tuple(max(1, (i + 2) // 4) for i in w.shape)
    g = synth.gradient(w, 0)
    errs = run(g, w.ranks, ranks25, w.k)
    text = report(errs, w.shape, w.ranks, ranks25, w.k)
    if args.out == "-":
        sys.stdout.write(text)
    else:
        with open(args.out, "w") as f:
            f.write(text)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
