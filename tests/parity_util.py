"""Step-by-step comparison of libefcp (GPU) with the CPU oracle on the same
float32 gradient bytes.  Bars (from the benchmark definition):
  * Top-k indices, stored values and the error-feedback buffer: bit-exact at
    every step;
  * F^-1 x: relative L2 error <= 1e-3 at every step (fp32 output against the
    oracle's fp64; observed errors are ~1e-7);
  * S, q: fp64 sums of exact products in a different order: 1e-10 relative to
    the largest magnitude involved;  coef is reported, not gated, because it is
    conditioning-dependent and the bar is on the output.
"""
from __future__ import annotations

import numpy as np

OUT_TOL = 1e-3


def bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint32)


def rel_l2(a: np.ndarray, ref: np.ndarray) -> float:
    den = np.linalg.norm(ref)
    num = np.linalg.norm(np.asarray(a, dtype=np.float64) - ref)
    return float(num / den) if den > 0 else float(num)


def run_parity(torch, oracle_mod, binding, d, m, k, lam, grads, check_error_every=1,
               check_small=True, verbose=False, out_tol=OUT_TOL, bf16=False,
               compressed=False, update=None, apply_every=0, topk_block=0, ggt=False, fill=0,
               fill_check_every=128, say=None, slice_width=0):
    """grads: iterable of float32 numpy arrays.  bf16: the bfloat16 window
    format on both sides.  compressed: the step preconditions c_t instead of
    the gradient.  update=(lr, weight_decay): the step updates a parameter
    vector in place instead of writing F^-1 x; the bar is then on the update,
    |theta_gpu - theta_ref| relative to |lr * F^-1 x|, with both sides starting
    each step from the same fp32 parameters.  apply_every=n: after every n-th
    step a seeded random x is applied to the window as it stands on both
    sides (no insertion).  topk_block=B: Top-k applied in blocks of B
    coordinates on both sides, k entries per block.  ggt: Sparse GGT on both
    sides, lam is its epsilon.  fill=n: the first n steps only insert on both
    sides (the oracle's step without output, out = NULL on the GPU): the new row
    is still compared bit for bit on every one of them, e and all of S on every
    fill_check_every-th and on the last; from step n+1 on every step is a full one.  say: callable for
    progress lines.  slice_width: d-slice width of the GPU context (0 = automatic).
    Returns dict of worst errors."""
    dev = torch.device("cuda:0")
    o = oracle_mod.Oracle(d, m, k, lam, values_bf16=bf16, block=topk_block, ggt=ggt)
    g_gpu = binding.Efcp(d, m, k, lam, values=binding.VALUES_BF16 if bf16 else binding.VALUES_FP32,
                         topk_block=topk_block, ggt=ggt, slice_width=slice_width)
    assert g_gpu.k == o.k, "row length differs"
    e_prev = np.zeros(d, np.float32)
    grad_d = torch.empty(d, dtype=torch.float32, device=dev)
    out_d = torch.empty(d, dtype=torch.float32, device=dev)
    worst = dict(out=0.0, S=0.0, q=0.0, coef=0.0, apply=0.0)
    rng = np.random.default_rng(d + m)
    theta = (rng.standard_normal(d) * 0.05).astype(np.float32) if update else None
    x_source = binding.X_COMPRESSED if compressed else binding.X_GRAD
    t = 0
    try:
        for g in grads:
            t += 1
            g = np.ascontiguousarray(g, dtype=np.float32)
            a = e_prev + g                      # the accumulator, one fp32 rounding per element
            filling = t <= fill
            if filling:
                o.step_no_output(g)
            else:
                y = o.step_compressed(g) if compressed else o.step(g)
            e_prev = o.error.copy()
            grad_d.copy_(torch.from_numpy(g))
            if filling:
                g_gpu.step(grad_d, None)
            elif update:
                out_d.copy_(torch.from_numpy(theta))
                g_gpu.step_ex(grad_d, x_source, param=out_d, lr=update[0], weight_decay=update[1])
            elif compressed:
                g_gpu.step_ex(grad_d, x_source, out=out_d)
            else:
                g_gpu.step(grad_d, out_d)
            torch.cuda.synchronize()
            slot = (t - 1) % m
            idx, val = g_gpu.get_row(slot)
            oi, ov = o.row(slot)
            assert np.array_equal(idx, oi), f"step {t}: Top-k indices differ"
            assert np.array_equal(bits(val), bits(ov)), f"step {t}: stored values differ"
            if filling:
                check_e = t == fill or t % fill_check_every == 0
            else:
                check_e = check_error_every and (t % check_error_every == 0 or t == 1)
            if check_e:
                assert np.array_equal(bits(g_gpu.get_error()), bits(o.error)), \
                    f"step {t}: error feedback differs"
            if filling:
                if check_e:
                    S_gpu, S_ref = g_gpu.get_small()["S"], o.gram
                    sS = np.abs(S_gpu - S_ref).max() / max(np.abs(S_ref).max(), 1e-300)
                    worst["S"] = max(worst["S"], sS)
                    assert sS <= 1e-10, f"step {t} (fill): Gram matrix off by {sS:.3e}"
                    if say:
                        say(f"fill step {t}/{fill}: rows, e bit-exact so far; S within {sS:.1e}")
                continue
            out = out_d.cpu().numpy()
            assert np.isfinite(out).all(), f"step {t}: non-finite output"
            if update:
                theta_ref = oracle_mod.param_update(theta, y, update[0], update[1])
                moved = np.linalg.norm(update[0] * y)
                err = float(np.linalg.norm(out.astype(np.float64) - theta_ref) / moved) if moved > 0 else 0.0
                theta = theta_ref
            else:
                err = rel_l2(out, y)
            worst["out"] = max(worst["out"], err)
            if out_tol is not None:
                assert err <= out_tol, f"step {t}: rel L2 of F^-1 x = {err:.3e}"
            if check_small:
                sm = g_gpu.get_small()
                assert sm["step"] == t
                S_ref, q_ref = o.gram, o.q
                sS = np.abs(sm["S"] - S_ref).max() / max(np.abs(S_ref).max(), 1e-300)
                sq = np.abs(sm["q"] - q_ref).max() / max(np.abs(q_ref).max(), 1e-300)
                sc = np.abs(sm["coef"] - o.coef).max() / max(np.abs(o.coef).max(), 1e-300)
                worst["S"] = max(worst["S"], sS)
                worst["q"] = max(worst["q"], sq)
                worst["coef"] = max(worst["coef"], sc)
                assert sS <= 1e-10, f"step {t}: Gram matrix off by {sS:.3e}"
                assert sq <= 1e-10, f"step {t}: q off by {sq:.3e}"
                if not topk_block:
                    sel_key = bits(a[oi]) & np.uint32(0x7FFFFFFF)
                    assert sm["tau"] == int(sel_key.min()), f"step {t}: threshold key differs"
            if apply_every and t % apply_every == 0:
                x = (rng.standard_normal(d) * np.exp(rng.standard_normal(d))).astype(np.float32)
                ya = o.apply(x)
                grad_d.copy_(torch.from_numpy(x))
                g_gpu.apply(grad_d, out_d)
                torch.cuda.synchronize()
                ea = rel_l2(out_d.cpu().numpy(), ya)
                worst["apply"] = max(worst["apply"], ea)
                assert ea <= OUT_TOL, f"step {t}: rel L2 of applied F^-1 x = {ea:.3e}"
                assert np.array_equal(bits(g_gpu.get_error()), bits(o.error)), f"step {t}: apply changed e"
                assert g_gpu.get_small()["step"] == t
            if verbose:
                print(f"  step {t}: out {err:.2e}", flush=True)
            if say:
                say(f"step {t}: rows, e bit-exact; out {err:.2e}")
    finally:
        g_gpu.destroy()
        o.close()
    worst["steps"] = t
    return worst
