"""GPU parity in the steady state: a FULL window that evicts its oldest row on
every step (Section "Efficient Full-Matrix Preconditioners": the ring buffer
replaces the oldest gradient; eq. (2) over the m rows present), checked
against the CPU oracle and nothing else.

* The ResNet-20-sized shape (d = 272,474, m = 1024, k = 2,725, lambda = 1e-5):
  1,024 insertion-only steps on both sides (every new row compared bit for
  bit), then full steps that evict, each compared like any other step: row and
  e bit-exact, all of S and q to 1e-10, F^-1 g to 1e-3.  This is the regime the
  benchmark times (m = 1024, one eviction per step), including the update of
  the inverse factor over all sixteen 64-row chunks.
* Windows of m in {65, 200, 1024} rows after many evictions (k = 64, and k = 3000 in slices of
  1024 coordinates so that the window passes run with 16 lanes per row): the rows are read
  back from the library, loaded into a FRESH oracle in age order, and the
  oracle's own Gram matrix (all of it) and F^-1 x for a new x are compared with
  the library's.  Nothing on the reference side comes from the library except
  the stored rows, which the step-by-step tests pin bit for bit.
"""
import time

import numpy as np
import pytest

from paper_2306_06098_amd import synth
from parity_util import rel_l2, run_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(oracle_mod):
    import torch
    from paper_2306_06098_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    return torch, oracle_mod, binding


def _sayer(capsys):
    def say(msg):
        with capsys.disabled():
            print(f"\n    [{time.strftime('%H:%M:%S')}] {msg}", flush=True)
    return say


def test_resnet20_shape_full_window_evicting_steps_vs_oracle(env, capsys):
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["resnet20"]
    evicting = 10
    s = synth.GradientStream(wl.d, wl.rho, wl.seed + 50)

    def grads():
        for _ in range(wl.m + evicting):
            yield s.next()
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, wl.k, wl.lam, grads(), fill=wl.m,
                   fill_check_every=128, check_small=True, say=_sayer(capsys))
    _sayer(capsys)(f"resnet20 shape, full window, {evicting} evicting steps: {w}")
    assert w["steps"] == wl.m + evicting


@pytest.mark.parametrize("bf16,slice_width", [(False, 0), (True, 0), (False, 8192), (True, 8192)])
def test_resnet20_shape_full_window_other_modes_vs_oracle(env, capsys, bf16, slice_width):
    """Same regime, fewer coordinates (the oracle's sort dominates the fill): bfloat16 window,
    and apply() on the full window after every evicting step.  With the automatic slice width a
    row has 5 entries per slice and the window passes give it 4 lanes; in slices of 8,192
    coordinates it has 78 and gets 16."""
    torch, oracle_mod, binding = env
    d, m, k, lam = 70_001, 1024, 700, 1e-5
    s = synth.GradientStream(d, 0.9, 77)

    def grads():
        for _ in range(m + 4):
            yield s.next()
    w = run_parity(torch, oracle_mod, binding, d, m, k, lam, grads(), fill=m, fill_check_every=256,
                   bf16=bf16, apply_every=1, say=_sayer(capsys), slice_width=slice_width)
    assert w["steps"] == m + 4


@pytest.mark.parametrize("m,steps,k,slice_width", [
    (65, 65 + 140, 64, 0), (200, 200 + 75, 64, 0), (1024, 1024 + 40, 64, 0),
    # 75 entries per row and slice: the window passes give a row 16 lanes (the cases above and the
    # ResNet-20 shape, with a dozen entries per row and slice, run them with 4)
    (1024, 1024 + 24, 3000, 1024),
])
def test_window_after_many_evictions_reloaded_into_a_fresh_oracle(env, m, steps, k, slice_width):
    torch, oracle_mod, binding = env
    d, lam = 40_003, 1e-4
    s = synth.GradientStream(d, 0.9, 21 + m)
    ctx = binding.Efcp(d, m, k, lam, slice_width=slice_width)
    g = torch.empty(d, dtype=torch.float32, device="cuda:0")
    out = torch.empty_like(g)
    for t in range(steps):
        x = s.next()
        g.copy_(torch.from_numpy(x))
        ctx.step(g, out)
    torch.cuda.synchronize()
    sm = ctx.get_small()
    assert sm["step"] == steps
    # age order, oldest first: the oracle that loads them in this order ends with the oldest in slot 0
    slots = [(steps - m + a) % m for a in range(m)]
    o = oracle_mod.Oracle(d, m, k, lam)
    for sl in slots:
        o.load_row(*ctx.get_row(sl))
    S_ref = o.gram                                  # by the fresh oracle's slots = by age
    S_gpu = sm["S"][np.ix_(slots, slots)]
    sS = np.abs(S_gpu - S_ref).max() / np.abs(S_ref).max()
    assert sS <= 1e-10, f"Gram matrix after {steps - m} evictions off by {sS:.3e}"
    # the last step's output, and a fresh x through apply(): both against the oracle's window
    y = o.apply(x)
    assert np.abs(sm["q"][slots] - o.q).max() <= 1e-10 * np.abs(o.q).max()
    e_step = rel_l2(out.cpu().numpy(), y)
    assert e_step <= 1e-3, f"F^-1 g of the last step off by {e_step:.3e}"
    rng = np.random.default_rng(m)
    x2 = (rng.standard_normal(d) * np.exp(rng.standard_normal(d))).astype(np.float32)
    y2 = o.apply(x2)
    g.copy_(torch.from_numpy(x2))
    ctx.apply(g, out)
    torch.cuda.synchronize()
    e_apply = rel_l2(out.cpu().numpy(), y2)
    assert e_apply <= 1e-3, f"apply() on the evicted-into window off by {e_apply:.3e}"
    sc = np.abs(ctx.get_small()["coef"][slots] - o.coef).max() / np.abs(o.coef).max()
    print(f"m={m}: S {sS:.1e}, step {e_step:.1e}, apply {e_apply:.1e}, coef {sc:.1e}")
    ctx.destroy()
    o.close()
