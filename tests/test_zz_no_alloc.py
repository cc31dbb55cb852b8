"""The allocation-free entry point `tgrad_step_static` against `tgrad_step`: same kernels, same
state layout, scratch in the library's fixed per-GPU array instead of a caller's workspace.  The
two must agree bit for bit (weights and every state item), on calls in a row that share the array:
a larger tensor, then a smaller one, then both again at t = 1 (no refresh: what a context keeps in
its workspace between steps has meanwhile been overwritten by the other tensor and must be
rebuilt), and so on across a second refresh."""
import numpy as np
import pytest

from paper_2501_02379_amd import synth
from paper_2501_02379_amd import tgrad as T

pytestmark = pytest.mark.gpu

CASES = [
    # shape, ranks, k, gradient dtype, weights, order            kernel tier
    ((16, 32, 64, 5), (4, 8, 16, 2), 200, "c64", "c64", 0),       # fused
    ((16, 16, 8, 5), (8, 8, 4, 3), 103, "c64", "c64", 0),         # matrix-core, unfused (the smaller input)
]
EXTRA = [
    ((12, 10, 9, 7), (3, 4, 2, 3), 60, "cbf16", "bf16", 0),       # half-precision gradients and weights
    ((8, 7, 40), (2, 2, 36), 30, "c64", "c64", 0),                # generic last-mode kernels (support bitmask)
    ((16, 32, 32, 9), (4, 8, 8, 4), 300, "c64", "c64", 1),        # low rank first, fused tier
]
ITEMS = [T.STATE_INDICES, T.STATE_CORE_M, T.STATE_CORE_V, T.STATE_SPARSE_M, T.STATE_SPARSE_V]


class _Job:
    """One tensor stepped both ways."""

    def __init__(self, shape, ranks, k, gdt, wdt, order, seed):
        import torch
        self.shape, self.gdt = shape, gdt
        self.cfg = T.make_config(shape, ranks, k, grad_dtype=T.TGRAD_CBF16 if gdt == "cbf16" else T.TGRAD_C64,
                                 weight_dtype=T.TGRAD_CBF16 if wdt == "bf16" else T.TGRAD_C64, lr=2e-3,
                                 weight_decay=0.01, refresh_every=3, order=order)
        self.ctx = T.Context(self.cfg)
        rng = np.random.default_rng(seed)
        W0 = ((rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * 0.02).astype(np.complex64)
        if wdt == "bf16":
            W0 = synth.complex64_to_bf16_pairs(W0)
        self.W_ctx = T.to_device_weight(W0)
        self.W_static = T.to_device_weight(W0)
        rc, sb, wb = T.tgrad_query_sizes(self.cfg)
        assert rc == T.TGRAD_OK and wb <= T.STATIC_WORKSPACE_BYTES
        self.state = torch.zeros(sb, dtype=torch.uint8, device="cuda:0")
        self.seed = seed
        self.t = 0

    def step(self):
        g = synth.small_case(self.shape, self.seed + 10 * self.t, dtype=self.gdt)
        gd = T.to_device_grad(g)
        self.ctx.tgrad_step(self.W_ctx, gd)
        T.tgrad_step_static(self.cfg, self.state, self.t, self.W_static, gd)
        self.t += 1

    def check(self):
        import torch
        torch.cuda.synchronize()
        assert np.array_equal(T.weight_to_host(self.W_static), T.weight_to_host(self.W_ctx)), ("weights", self.shape, self.t)
        # the static call's state buffer has the layout of a context's: compare the raw bytes
        a = self.state.cpu().numpy()
        b = self.ctx.state_buf.cpu().numpy()
        assert np.array_equal(a, b), ("state", self.shape, self.t)
        for it in ITEMS:
            assert self.ctx.tgrad_get_state(it) is not None


def test_static_step_matches_context_step_two_calls_in_a_row():
    big = _Job(*CASES[0], seed=4100)
    small = _Job(*CASES[1], seed=4200)
    big.step()                       # first call: the larger tensor, t = 0 (refresh inside)
    big.check()
    small.step()                     # second call in a row: a smaller tensor on the same array
    small.check()
    for _ in range(4):               # t = 1 .. 4, interleaved: steps without and with a refresh (t = 3)
        big.step()
        small.step()
        big.check()
        small.check()
    assert big.t == 5 and small.t == 5


@pytest.mark.parametrize("case", EXTRA)
def test_static_step_other_tiers_interleaved(case):
    a = _Job(*case, seed=4300)
    b = _Job(*CASES[1], seed=4400)
    for _ in range(5):
        a.step()
        b.step()
        a.check()
        b.check()


def test_static_step_rejects_what_it_cannot_serve():
    import ctypes as C
    import torch
    lib = T.load()
    w = synth.WORKLOADS["cfg3"]
    cfg = T.make_config(w.shape, w.ranks, w.k, refresh_every=w.T)
    rc, sb, wb = T.tgrad_query_sizes(cfg)
    assert rc == T.TGRAD_OK and wb > T.STATIC_WORKSPACE_BYTES
    dummy = torch.zeros(1024, dtype=torch.uint8, device="cuda:0")
    # too large for the fixed array: refused before anything is launched or dereferenced
    rc = lib.tgrad_step_static(C.byref(cfg), dummy.data_ptr(), 0, dummy.data_ptr() + 256, dummy.data_ptr() + 512, None)
    assert rc == T.TGRAD_ERR_UNSUPPORTED
    small = T.make_config((16, 16, 8, 5), (8, 8, 4, 3), 103, refresh_every=0)
    rc = lib.tgrad_step_static(C.byref(small), dummy.data_ptr(), 0, dummy.data_ptr() + 256, dummy.data_ptr() + 512, None)
    assert rc == T.TGRAD_ERR_INVALID_ARG           # no refresh period: nobody could refresh this state
    small = T.make_config((16, 16, 8, 5), (8, 8, 4, 3), 103, refresh_every=5)
    rc = lib.tgrad_step_static(C.byref(small), dummy.data_ptr(), -1, dummy.data_ptr() + 256, dummy.data_ptr() + 512, None)
    assert rc == T.TGRAD_ERR_INVALID_ARG
    rc = lib.tgrad_step_static(C.byref(small), None, 0, dummy.data_ptr() + 256, dummy.data_ptr() + 512, None)
    assert rc == T.TGRAD_ERR_INVALID_ARG
