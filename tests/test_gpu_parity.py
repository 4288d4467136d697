"""GPU parity tests: libefcp through its C ABI against the CPU oracle, same
float32 inputs, element by element (see parity_util for the bars)."""
import numpy as np
import pytest

from paper_2306_06098_amd import synth
from parity_util import bits, rel_l2, run_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(oracle_mod):
    import torch
    from paper_2306_06098_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()          # raises if libefcp.so was not built: no fallback
    return torch, oracle_mod, binding


def _stream(wl, T):
    s = synth.GradientStream(wl.d, wl.rho, wl.seed)
    for _ in range(T):
        yield s.next()


def test_tiny_workload_all_steps(env):
    """d=65,536, m=32, k=655, lambda=1e-4, 200 steps: window fills at step 32 and
    then evicts on every step."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["tiny"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, wl.k, wl.lam, _stream(wl, wl.T))
    print("tiny", w)
    assert w["steps"] == wl.T


def test_tiny_workload_all_steps_bf16_window(env):
    """Same workload with the bfloat16 window format (bf16 values, 16-bit
    in-slice indices): stored values, indices, e (with the rounding remainders)
    bit-exact against the oracle in the same mode; F^-1 g within 1e-3."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["tiny"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, wl.k, wl.lam, _stream(wl, wl.T), bf16=True)
    print("tiny bf16", w)
    assert w["steps"] == wl.T


def test_resnet20_workload_bf16_window(env):
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["resnet20"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, wl.k, wl.lam, _stream(wl, 120),
                   check_error_every=10, bf16=True)
    print("resnet20 bf16", w)


def test_resnet20_workload_all_steps(env):
    """d=272,474 (not a multiple of the slice, the compaction block or 4), m=1024,
    k=2,725, lambda=1e-5, 500 steps."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["resnet20"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, wl.k, wl.lam, _stream(wl, wl.T),
                   check_error_every=25)
    print("resnet20", w)
    assert w["steps"] == wl.T


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("d,m,k,lam,T", [
    (20_001, 8, 201, 1e-3, 40),       # ragged tail, eviction from step 9 on
    (4_099, 3, 4_099, 1e-2, 9),       # k = d: Dense M-FAC, e stays 0
    (70_000, 5, 1, 1e-2, 12),         # k = 1
    (3, 2, 2, 1e-1, 6),               # smaller than one vector load
    (16_384 * 3, 7, 500, 1e-4, 20),   # exact multiple of the slice
    (100_003, 1, 1000, 1e-3, 5),      # m = 1: every step evicts
])
def test_shapes_and_edges(env, d, m, k, lam, T, bf16):
    torch, oracle_mod, binding = env
    rng = np.random.default_rng(d + m)
    scale = np.exp(rng.standard_normal(d)).astype(np.float32)

    def grads():
        z = np.zeros(d, np.float32)
        for _ in range(T):
            z = (0.7 * z + rng.standard_normal(d)).astype(np.float32)
            yield scale * z
    w = run_parity(torch, oracle_mod, binding, d, m, k, lam, grads(), bf16=bf16)
    print((d, m, k, bf16), w)


@pytest.mark.parametrize("width", [256, 1024, 4352, 12_544, 15_936, 16_384])
@pytest.mark.parametrize("bf16", [False, True])
def test_slice_widths(env, width, bf16):
    """The d-slice width is an option of the context (efcp_options.slice_width): slices of 256 up to 16,384
    coordinates, widths that end in the middle of a wave's part of a block, in the middle of a
    4,096-coordinate chunk and (15,936) in the middle of a wave's 256-coordinate piece, d not a
    multiple of any of them; every variant of the step."""
    torch, oracle_mod, binding = env
    d, m, k, lam, T = 150_011, 6, 1_500, 1e-3, 14
    rng = np.random.default_rng(width)
    scale = np.exp(rng.standard_normal(d)).astype(np.float32)

    def grads():
        z = np.zeros(d, np.float32)
        for _ in range(T):
            z = (0.7 * z + rng.standard_normal(d)).astype(np.float32)
            yield scale * z
    g = binding.Efcp(d, m, k, lam, slice_width=width)
    geo = g.geometry()
    g.destroy()
    assert geo["slice"] == width and geo["n_slices"] == -(-d // width)
    w = run_parity(torch, oracle_mod, binding, d, m, k, lam, grads(), bf16=bf16, apply_every=5,
                   slice_width=width)
    w2 = run_parity(torch, oracle_mod, binding, d, m, k, lam, grads(), bf16=bf16, compressed=True,
                    update=(0.05, 0.01), slice_width=width)
    print(width, bf16, w, w2)


def test_slice_width_is_chosen_from_d(env):
    """Automatic width: short vectors are cut into (up to) 256 slices of at least 1,024
    coordinates (a multiple of 256); longer ones into nearly equal slices (a multiple of 64) that
    fill every round of 256 workgroups when rounds of widest slices would be at least 2 % empty,
    else into widest slices; Top-k in blocks keeps the block."""
    torch, oracle_mod, binding = env
    for d, kw, want in [(5_000, {}, 1024), (272_474, {}, 1280), (11_200_000, {}, 14_592),
                        (4_194_304, {}, 16_384), (4_194_305, {}, 8_256),
                        (21_100_000, {}, 13_760), (110_000_000, {}, 15_936), (340_000_000, {}, 16_384),
                        (272_474, dict(topk_block=binding.TOPK_BLOCK), 16_384)]:
        g = binding.Efcp(d, 2, 3, 1e-3, **kw)
        geo = g.geometry()
        g.destroy()
        assert geo["slice"] == want and geo["n_slices"] == -(-d // want), (d, geo)


def test_random_shapes_sweep(env):
    """Thirty seeded random (d, m, k, lambda) with d from a handful of elements to
    several slices plus a ragged tail, k from 1 to d, windows that fill and evict;
    some streams quantised to force ties at the threshold."""
    torch, oracle_mod, binding = env
    rng = np.random.default_rng(2024)
    for case in range(30):
        d = int(rng.choice([rng.integers(1, 64), rng.integers(64, 5_000), rng.integers(5_000, 140_000)]))
        m = int(rng.integers(1, 24))
        k = int(rng.choice([1, d, rng.integers(1, d + 1), max(1, d // 100)]))
        lam = float(10.0 ** rng.uniform(-5, 0))
        T = m + int(rng.integers(1, 8))
        quant = case % 3 == 0
        scale = np.exp(rng.standard_normal(d)).astype(np.float32)

        def grads():
            z = np.zeros(d, np.float32)
            for _ in range(T):
                z = (0.8 * z + rng.standard_normal(d)).astype(np.float32)
                g = scale * z
                yield (np.round(g * 4) / 4).astype(np.float32) if quant else g
        w = run_parity(torch, oracle_mod, binding, d, m, k, lam, grads(), bf16=case % 2 == 1)
        print(case, (d, m, k, lam, T, quant), w["out"])


@pytest.mark.parametrize("topk_block", [0, 16_384])
def test_non_finite_gradient_entries_are_ordered_by_their_bits(env, topk_block):
    """Infinities and NaN are not rejected: their magnitude keys (0x7f800000, 0x7fc00000) sort
    above every finite value, so they are selected like any other large entry, e = a - c makes
    them NaN, and later steps select those again.  Indices must agree exactly; values and e
    bit for bit except that any NaN matches any NaN (the two machines sign the NaN of inf - inf
    differently).  The preconditioned output is meaningless from then on and is not looked at."""
    torch, oracle_mod, binding = env
    d, m, lam = 50_003, 4, 1e-3
    k = 40 if topk_block else 500
    rng = np.random.default_rng(77)
    o = oracle_mod.Oracle(d, m, k, lam, block=topk_block)
    ctx = binding.Efcp(d, m, k, lam, topk_block=topk_block)
    g_d = torch.empty(d, dtype=torch.float32, device="cuda:0")
    out_d = torch.empty_like(g_d)

    def same(a, b):
        a, b = np.asarray(a, np.float32), np.asarray(b, np.float32)
        return bool(np.all((bits(a) == bits(b)) | (np.isnan(a) & np.isnan(b))))
    try:
        for t in range(6):
            g = rng.standard_normal(d).astype(np.float32)
            if t == 2:
                g[100], g[20_000], g[33_333] = np.inf, -np.inf, np.float32(np.nan)
            o.step(g)
            g_d.copy_(torch.from_numpy(g))
            ctx.step(g_d, out_d)
            torch.cuda.synchronize()
            slot = t % m
            idx, val = ctx.get_row(slot)
            oi, ov = o.row(slot)
            assert np.array_equal(idx, oi), f"step {t + 1}: indices differ"
            assert same(val, ov), f"step {t + 1}: values differ"
            assert same(ctx.get_error(), o.error), f"step {t + 1}: error feedback differs"
            if t >= 2:
                assert np.isin([100, 20_000, 33_333], idx).all()
    finally:
        ctx.destroy()
        o.close()


def test_forced_ties_integer_gradients(env):
    """Small-integer gradients: the threshold magnitude is shared by many
    coordinates on every step, so the lowest-index tie rule decides."""
    torch, oracle_mod, binding = env
    d, m, k = 50_001, 5, 500
    it = synth.integer_stream(d, seed=9)
    w = run_parity(torch, oracle_mod, binding, d, m, k, 1e-2, (next(it) for _ in range(15)))
    print("ties", w)
    it = synth.integer_stream(d, seed=10, lo=-700, hi=700)
    w = run_parity(torch, oracle_mod, binding, d, m, k, 1e-2, (next(it) for _ in range(15)), bf16=True)
    print("ties bf16", w)


def test_threshold_jumps_between_steps(env):
    """The candidate filter of the first pass is seeded by the previous step's
    threshold.  Make the threshold collapse by orders of magnitude (the later
    passes then read the accumulator instead of the candidate lists), stay put, and jump up again; with k < d and
    with k = d (no residual left in e)."""
    torch, oracle_mod, binding = env
    rng = np.random.default_rng(77)
    # the last shape: 245 slices, i.e. 16 workgroups of 16 segments in the passes that fall back to
    # the accumulator, a ragged last slice, and the bfloat16 window
    for d, m, k, bf16 in ((60_000, 6, 600, False), (20_000, 4, 20_000, False), (1_000_003, 5, 10_000, False),
                          (1_000_003, 5, 10_000, True)):
        base = rng.standard_normal(d).astype(np.float32)
        probe = oracle_mod.Oracle(d, m, k, 1e-2)
        probe.step(base)
        resid = probe.error.copy()            # what is left below the first threshold
        noise = [rng.standard_normal(d).astype(np.float32) for _ in range(8)]
        grads = [base,
                 (-resid + 1e-4 * noise[0]).astype(np.float32),     # a ~ 1e-4: collapse
                 (1e-4 * noise[1]).astype(np.float32),              # stays small
                 (1e-9 * noise[2]).astype(np.float32),              # collapses again (k = d) or rides on e
                 (50.0 * noise[3]).astype(np.float32),              # jumps up
                 (1e-2 * noise[4]).astype(np.float32),
                 noise[5], (3e-3 * noise[6]).astype(np.float32), noise[7]]
        w = run_parity(torch, oracle_mod, binding, d, m, k, 1e-2, grads, bf16=bf16)
        print("jumps", (d, m, k, bf16), w)


def test_degenerate_vectors(env):
    """All-equal, all-zero (with signed zeros), subnormal and huge values: the
    bit-exact part (Top-k, stored values, error feedback, threshold key) is what
    this test is for.  The output is only required to be finite here: with
    entries of 3e30 next to entries of 1 in one row, x/lambda - sum cancels
    totally at the huge coordinates and even the fp64 oracle keeps no correct
    digit there, so a relative-L2 bar on F^-1 x is meaningless for this input."""
    torch, oracle_mod, binding = env
    d, m, k = 30_000, 4, 300
    tiny = np.float32(1e-45)
    g0 = np.full(d, 2.5, np.float32)
    g1 = np.zeros(d, np.float32); g1[::3] = -0.0
    g2 = np.full(d, tiny, np.float32); g2[::7] = -2 * tiny; g2[5] = 1e-38
    g3 = np.zeros(d, np.float32); g3[d - 1] = 3e30; g3[0] = -3e30; g3[1:400] = 1.0
    # zero first so that signed zeros survive in e; all-equal next
    w = run_parity(torch, oracle_mod, binding, d, m, k, 1e-2, [g1, g1, g0, g2, g3, g0, g1],
                   out_tol=None)
    print("degenerate", w)


def test_determinism_bitwise(env):
    torch, _, binding = env
    wl = synth.WORKLOADS["tiny"]
    outs = []
    for _ in range(2):
        ctx = binding.Efcp(wl.d, wl.m, wl.k, wl.lam)
        g = torch.empty(wl.d, dtype=torch.float32, device="cuda:0")
        out = torch.empty_like(g)
        acc = []
        for x in _stream(wl, 50):
            g.copy_(torch.from_numpy(x))
            ctx.step(g, out)
            acc.append(out.cpu().numpy().copy())
        ctx.destroy()
        outs.append(acc)
    for a, b in zip(*outs):
        assert np.array_equal(bits(a), bits(b))


def test_full_1024_window_factor_update(env):
    """m = 1024 with eviction, which the oracle cannot reach in seconds: after
    1,060 steps the coefficients must solve (m*lambda*I + S) coef = q/lambda for
    the library's own S and q (both validated against the oracle elsewhere), and
    out must equal x/lambda - sum coef_r c_r rebuilt from the exported rows."""
    torch, _, binding = env
    d, m, k, lam = 40_003, 1024, 64, 1e-4
    s = synth.GradientStream(d, 0.9, 21)
    ctx = binding.Efcp(d, m, k, lam)
    g = torch.empty(d, dtype=torch.float32, device="cuda:0")
    out = torch.empty_like(g)
    for t in range(1060):
        x = s.next()
        g.copy_(torch.from_numpy(x))
        ctx.step(g, out)
    sm = ctx.get_small()
    A = m * lam * np.eye(m) + sm["S"]
    ref = np.linalg.solve(A, sm["q"]) / lam
    assert rel_l2(sm["coef"], ref) < 1e-8
    y = x.astype(np.float64) / lam
    for r in range(m):
        i, v = ctx.get_row(r)
        y[i] -= ref[r] * v.astype(np.float64)
    assert rel_l2(out.cpu().numpy(), y) < 1e-5
    ctx.destroy()


def test_inverse_factor_does_not_drift(env):
    """3,000 steps with a 16-slot window: 2,984 evictions applied to the
    inverse factor one after another.  The coefficients must still solve
    (m*lambda*I + S) coef = q/lambda for the current S and q."""
    torch, _, binding = env
    d, m, k, lam = 4_096, 16, 41, 1e-5
    s = synth.GradientStream(d, 0.95, 33)
    ctx = binding.Efcp(d, m, k, lam)
    g = torch.empty(d, dtype=torch.float32, device="cuda:0")
    out = torch.empty_like(g)
    worst = 0.0
    for t in range(1, 3001):
        g.copy_(torch.from_numpy(s.next()))
        ctx.step(g, out)
        if t % 500 == 0:
            sm = ctx.get_small()
            ref = np.linalg.solve(m * lam * np.eye(m) + sm["S"], sm["q"]) / lam
            worst = max(worst, rel_l2(sm["coef"], ref))
    print("drift", worst)
    assert worst < 1e-8
    ctx.destroy()


def test_steps_without_output_update_the_same_state(env):
    """out = NULL skips only the LCG pass: window, e, S, q, coef and every later
    output are bit-identical to a run that asked for the output on each step."""
    torch, _, binding = env
    d, m, k, lam = 50_000, 6, 500, 1e-3
    grads = list(_stream(synth.Workload("x", d, m, k, lam, 14, 0.9, 5), 14))
    res = []
    for skip in (False, True):
        ctx = binding.Efcp(d, m, k, lam)
        g = torch.empty(d, dtype=torch.float32, device="cuda:0")
        out = torch.full((d,), 7.0, dtype=torch.float32, device="cuda:0")
        for t, x in enumerate(grads):
            g.copy_(torch.from_numpy(x))
            ctx.step(g, None if (skip and t < 10) else out)
            if skip and t == 9:
                assert bool((out == 7.0).all())          # never written so far
        sm = ctx.get_small()
        res.append((out.cpu().numpy().copy(), ctx.get_error(), sm["S"], sm["q"], sm["coef"],
                    [ctx.get_row(r) for r in range(m)]))
        ctx.destroy()
    a, b = res
    assert np.array_equal(bits(a[0]), bits(b[0])) and np.array_equal(bits(a[1]), bits(b[1]))
    for i in (2, 3, 4):
        assert np.array_equal(a[i], b[i])
    for (i0, v0), (i1, v1) in zip(a[5], b[5]):
        assert np.array_equal(i0, i1) and np.array_equal(bits(v0), bits(v1))


def test_export_import_resumes_bit_identically(env):
    """Checkpoint in the middle of a run (partly filled window, then an evicting
    one), import into a fresh context, continue both: same bits everywhere."""
    torch, _, binding = env
    d, m, k, lam = 70_001, 7, 650, 1e-3
    grads = list(_stream(synth.Workload("x", d, m, k, lam, 24, 0.9, 8), 24))
    g = torch.empty(d, dtype=torch.float32, device="cuda:0")
    for cut, values in ((4, binding.VALUES_FP32), (15, binding.VALUES_FP32), (15, binding.VALUES_BF16)):
        a = binding.Efcp(d, m, k, lam, values=values)
        out_a = torch.empty_like(g)
        for x in grads[:cut]:
            g.copy_(torch.from_numpy(x)); a.step(g, out_a)
        blob = a.export_state()
        b = binding.Efcp(d, m, k, lam, values=values)
        b.import_state(blob)
        assert b.get_small()["step"] == cut
        out_b = torch.empty_like(g)
        for x in grads[cut:]:
            g.copy_(torch.from_numpy(x)); a.step(g, out_a); b.step(g, out_b)
            assert bool((out_a.view(torch.int32) == out_b.view(torch.int32)).all())
        assert np.array_equal(bits(a.get_error()), bits(b.get_error()))
        sa, sb = a.get_small(), b.get_small()
        assert np.array_equal(sa["S"], sb["S"]) and np.array_equal(sa["coef"], sb["coef"])
        for r in range(m):
            (i0, v0), (i1, v1) = a.get_row(r), b.get_row(r)
            assert np.array_equal(i0, i1) and np.array_equal(bits(v0), bits(v1))
        # a context of another shape refuses the blob; a truncated blob is refused too
        c = binding.Efcp(d, m, k + 1, lam, values=values)
        with pytest.raises(binding.EfcpError):
            c.import_state(blob)
        c.destroy()
        c = binding.Efcp(d, m, k, lam, values=1 - values)          # other window format
        with pytest.raises(binding.EfcpError):
            c.import_state(blob)
        with pytest.raises(binding.EfcpError):
            b.import_state(blob[: blob.size // 2])
        for ctx in (a, b, c):
            ctx.destroy()
    # a context cut into slices of another width refuses the blob as well
    c = binding.Efcp(d, m, k, lam, values=binding.VALUES_BF16, slice_width=2048)
    with pytest.raises(binding.EfcpError):
        c.import_state(blob)
    c.destroy()


def test_argument_checks(env):
    torch, _, binding = env
    for bad in [(0, 4, 1, 1e-3), (100, 0, 10, 1e-3), (100, 1025, 10, 1e-3), (100, 4, 101, 1e-3),
                (100, 4, 10, 0.0), (100, 4, 10, float("nan")), (2 ** 31, 4, 10, 1e-3)]:
        with pytest.raises(binding.EfcpError) as ei:
            binding.Efcp(*bad)
        assert ei.value.code == binding.EFCP_EINVAL
    for width in (-256, 1, 128, 255, 1000, 16_640, 32_768):         # not a multiple of 64 in [256, 16384]
        with pytest.raises(binding.EfcpError) as ei:
            binding.Efcp(100_000, 4, 10, 1e-3, slice_width=width)
        assert ei.value.code == binding.EFCP_EINVAL
        assert binding.efcp_workspace_bytes(100_000, 4, 10, slice_width=width) == 0
    with pytest.raises(binding.EfcpError):                          # 2^30 / 256 slices: too many per workgroup
        binding.Efcp(2 ** 30, 1, 10, 1e-3, slice_width=256)
    assert binding.efcp_workspace_bytes(100_000, 4, 10, slice_width=512) > 0
    ctx = binding.Efcp(1000, 4, 10, 1e-3)
    g = torch.zeros(1004, dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.EfcpError):
        ctx.step_ptr(g.data_ptr(), g.data_ptr(), 0)                 # aliasing
    with pytest.raises(binding.EfcpError):
        ctx.step_ptr(g.data_ptr() + 4, g.data_ptr() + 4096, 0)      # misaligned
    with pytest.raises(binding.EfcpError):
        ctx.get_row(0)                                              # not filled yet
    ctx.destroy()


# ---------------------------------------------------------------------------
# efcp_step_ex / efcp_apply: other vectors through the same window

def _edge_grads(d, T, seed):
    rng = np.random.default_rng(seed)
    scale = np.exp(rng.standard_normal(d)).astype(np.float32)
    z = np.zeros(d, np.float32)
    for _ in range(T):
        z = (0.7 * z + rng.standard_normal(d)).astype(np.float32)
        yield scale * z


@pytest.mark.parametrize("bf16", [False, True])
def test_compressed_accumulator_is_preconditioned(env, bf16):
    """x = c_t (Algorithm 1 line 8 as printed): F^-1 c_t against the oracle on
    the tiny workload, state bit-exact as in the x = g mode."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["tiny"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, wl.k, wl.lam, _stream(wl, 80), bf16=bf16,
                   compressed=True)
    print("tiny compressed", bf16, w)


@pytest.mark.parametrize("d,m,k,lam,T", [(20_001, 8, 201, 1e-3, 30), (4_099, 3, 4_099, 1e-2, 9),
                                          (16_384 * 3, 7, 500, 1e-4, 16), (100_003, 1, 1000, 1e-3, 5),
                                          (3, 2, 2, 1e-1, 6)])
def test_compressed_mode_shapes(env, d, m, k, lam, T):
    torch, oracle_mod, binding = env
    w = run_parity(torch, oracle_mod, binding, d, m, k, lam, _edge_grads(d, T, d + m), compressed=True)
    print((d, m, k), w)


@pytest.mark.parametrize("compressed", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
def test_fused_parameter_update(env, bf16, compressed):
    """theta <- (1 - lr*wd)*theta - lr*F^-1 x inside the LCG kernel, against the
    oracle's fp64 update of the same fp32 parameters."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["tiny"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, wl.k, wl.lam, _stream(wl, 60), bf16=bf16,
                   compressed=compressed, update=(3e-6, 0.01))
    print("tiny update", bf16, compressed, w)
    # ragged last slice and a window that evicts
    d, m, k = 50_001, 4, 300
    w = run_parity(torch, oracle_mod, binding, d, m, k, 1e-3, _edge_grads(d, 10, 5), bf16=bf16,
                   compressed=compressed, update=(1e-4, 0.1))
    print("ragged update", bf16, compressed, w)


@pytest.mark.parametrize("bf16", [False, True])
def test_apply_on_fixed_window(env, bf16):
    """efcp_apply between steps: arbitrary dense x, partly filled and wrapped
    windows, nothing in the state moves (later steps still match bit for bit)."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["tiny"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, wl.k, wl.lam, _stream(wl, 70), bf16=bf16,
                   apply_every=3)
    print("tiny apply", bf16, w)
    assert w["apply"] > 0.0
    d, m, k = 40_003, 5, 77
    w = run_parity(torch, oracle_mod, binding, d, m, k, 1e-2, _edge_grads(d, 12, 9), bf16=bf16, apply_every=1)
    print("ragged apply", bf16, w)


def test_apply_before_first_step_and_repeats(env):
    """Empty window: F = lambda*I.  Two applies of the same x give the same bits,
    and apply(g) right after step(g) repeats the step's output bit for bit."""
    torch, oracle_mod, binding = env
    d, m, k, lam = 30_011, 6, 150, 1e-3
    dev = torch.device("cuda:0")
    o = oracle_mod.Oracle(d, m, k, lam)
    g_gpu = binding.Efcp(d, m, k, lam)
    try:
        rng = np.random.default_rng(3)
        x = rng.standard_normal(d).astype(np.float32)
        x_d = torch.from_numpy(x).to(dev)
        out_d = torch.empty_like(x_d)
        g_gpu.apply(x_d, out_d)
        torch.cuda.synchronize()
        assert rel_l2(out_d.cpu().numpy(), o.apply(x)) < 1e-6
        step_out = torch.empty_like(x_d)
        for t in range(9):
            g = rng.standard_normal(d).astype(np.float32)
            g_d = torch.from_numpy(g).to(dev)
            o.step(g)
            g_gpu.step(g_d, step_out)
            g_gpu.apply(g_d, out_d)
            again = torch.empty_like(out_d)
            g_gpu.apply(g_d, again)
            torch.cuda.synchronize()
            assert torch.equal(out_d, again)
            assert rel_l2(out_d.cpu().numpy(), o.apply(g)) <= 1e-3
            # same window, same x: q has a different summation order than in the step, so
            # the outputs agree to rounding, not necessarily bit for bit
            assert rel_l2(out_d.cpu().numpy(), step_out.cpu().numpy().astype(np.float64)) < 1e-5
    finally:
        g_gpu.destroy()
        o.close()


def test_step_ex_argument_checks(env):
    torch, oracle_mod, binding = env
    d = 5000
    dev = torch.device("cuda:0")
    g_gpu = binding.Efcp(d, 4, 50, 1e-2)
    try:
        g = torch.zeros(d, device=dev)
        a = torch.zeros(d, device=dev)
        b = torch.zeros(d, device=dev)
        with pytest.raises(binding.EfcpError):
            g_gpu.step_ex(g, binding.X_GRAD, out=a, param=b, lr=0.1)       # both destinations
        with pytest.raises(binding.EfcpError):
            g_gpu.step_ex(g, 7, out=a)                                      # unknown source
        with pytest.raises(binding.EfcpError):
            g_gpu.step_ex(g, binding.X_GRAD, param=a, lr=float("nan"))
        with pytest.raises(binding.EfcpError):
            g_gpu.apply(g, g)                                               # overlap
        assert g_gpu.get_small()["step"] == 0                               # nothing ran
    finally:
        g_gpu.destroy()


# ---------------------------------------------------------------------------
# Top-k applied in blocks of 16,384 coordinates (Section "Sparsity Pattern")

@pytest.mark.parametrize("bf16", [False, True])
def test_blockwise_topk_tiny_workload(env, bf16):
    """d = 65,536 = 4 blocks, 164 entries kept per block (1 %), all 200 steps."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["tiny"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, 164, wl.lam, _stream(wl, wl.T), bf16=bf16,
                   topk_block=binding.TOPK_BLOCK)
    print("tiny blockwise", bf16, w)
    assert w["steps"] == wl.T


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("d,m,kb,lam,T", [
    (272_474, 16, 164, 1e-5, 30),     # 16 full blocks + a ragged one of 10,330 coordinates
    (16_384 * 3, 7, 1, 1e-4, 12),     # one entry per block
    (16_384 + 1, 3, 16_384, 1e-2, 7),  # every coordinate kept: e stays 0; tail block of one element
    (20_001, 5, 4099, 1e-3, 11),      # large share, ragged
    (3, 2, 5000, 1e-1, 6),            # a single tiny block: keeps ceil(5000*3/16384) = 1
    (100_003, 1, 333, 1e-3, 5),       # m = 1
])
def test_blockwise_topk_shapes(env, d, m, kb, lam, T, bf16):
    torch, oracle_mod, binding = env
    w = run_parity(torch, oracle_mod, binding, d, m, kb, lam, _edge_grads(d, T, d + m), bf16=bf16,
                   topk_block=binding.TOPK_BLOCK, apply_every=4)
    print((d, m, kb, bf16), w)


def test_blockwise_topk_ties_and_threshold_jumps(env):
    """Integer gradients (ties at every block's threshold), then blocks whose
    magnitudes collapse and explode between steps (the per-block starting bin of
    the first histogram is then wrong and the kernel must recount)."""
    torch, oracle_mod, binding = env
    d, m, kb = 70_000, 6, 200
    s = synth.integer_stream(d, seed=21)
    w = run_parity(torch, oracle_mod, binding, d, m, kb, 1e-2, (next(s) for _ in range(25)),
                   topk_block=binding.TOPK_BLOCK)
    print("blockwise ties", w)
    rng = np.random.default_rng(22)

    def jumps():
        for t in range(16):
            g = rng.standard_normal(d).astype(np.float32)
            scale = np.ones(d, np.float32)
            for b in range(0, d, 16_384):
                scale[b:b + 16_384] = np.float32(10.0 ** rng.integers(-8, 8))
            yield g * scale
    w = run_parity(torch, oracle_mod, binding, d, m, kb, 1e-2, jumps(), topk_block=binding.TOPK_BLOCK,
                   out_tol=None)
    print("blockwise jumps", w)


def test_blockwise_topk_modes_and_checkpoint(env):
    """x = c_t and the fused update on a block-wise window; export / import."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["tiny"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, 164, wl.lam, _stream(wl, 50),
                   topk_block=binding.TOPK_BLOCK, compressed=True, update=(3e-6, 0.01))
    print("tiny blockwise compressed update", w)
    d, m, kb, lam = 50_001, 4, 100, 1e-3
    dev = torch.device("cuda:0")
    a = binding.Efcp(d, m, kb, lam, topk_block=binding.TOPK_BLOCK)
    b = binding.Efcp(d, m, kb, lam, topk_block=binding.TOPK_BLOCK)
    c = binding.Efcp(d, m, a.k, lam)                      # same row length, global Top-k
    try:
        grads = [torch.from_numpy(g).to(dev) for g in _edge_grads(d, 9, 77)]
        oa, ob = torch.empty(d, device=dev), torch.empty(d, device=dev)
        for g in grads[:6]:
            a.step(g, oa)
        blob = a.export_state()
        with pytest.raises(binding.EfcpError):
            c.import_state(blob)                          # selection rule is part of the state's shape
        b.import_state(blob)
        for g in grads[6:]:
            a.step(g, oa)
            b.step(g, ob)
            torch.cuda.synchronize()
            assert torch.equal(oa, ob)
        assert np.array_equal(bits(a.get_error()), bits(b.get_error()))
        with pytest.raises(binding.EfcpError):
            binding.Efcp(d, m, kb, lam, topk_block=4096)  # only the slice width is supported
        with pytest.raises(binding.EfcpError):
            binding.Efcp(d, m, 16_385, lam, topk_block=binding.TOPK_BLOCK)
    finally:
        a.destroy(); b.destroy(); c.destroy()


# ---------------------------------------------------------------------------
# Sparse GGT on the same window (Appendix "Sparse GGT")

@pytest.mark.parametrize("bf16", [False, True])
def test_sparse_ggt_tiny_workload(env, bf16):
    """d = 65,536, m = 32, k = 655, epsilon = 1e-2: the paper's variant
    (x = c_t) for 120 steps, with an apply of a random x after every fifth."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["tiny"]
    w = run_parity(torch, oracle_mod, binding, wl.d, wl.m, wl.k, 1e-2, _stream(wl, 120), bf16=bf16,
                   ggt=True, compressed=True, apply_every=5)
    print("tiny ggt", bf16, w)
    assert w["steps"] == 120 and w["apply"] > 0.0


def test_sparse_ggt_resnet20_sized(env):
    """The paper's GGT setting: d = 272,474 (ResNet-20), m = 100, 1 % density.  The window fills
    at step 100 and then evicts."""
    torch, oracle_mod, binding = env
    wl = synth.WORKLOADS["resnet20"]
    w = run_parity(torch, oracle_mod, binding, wl.d, 100, wl.k, 1e-3, _stream(wl, 112), ggt=True,
                   compressed=True, check_error_every=20)
    print("resnet20 ggt", w)


@pytest.mark.parametrize("d,m,k,eps,T,kw", [
    (20_001, 8, 201, 1e-3, 24, dict()),                         # x = g
    (20_001, 7, 201, 1e-2, 20, dict(update=(1e-3, 0.05))),      # odd m (dummy player), fused update
    (4_099, 3, 4_099, 1e-1, 9, dict(compressed=True)),          # k = d
    (70_000, 128, 40, 1e-2, 140, dict(compressed=True)),        # largest window; fills, then evicts
    (3, 2, 2, 1e-1, 6, dict()),
    (100_003, 1, 1000, 1e-3, 5, dict(compressed=True)),         # m = 1
    (50_000, 6, 100, 1e-2, 14, dict(topk_block=16_384, apply_every=2)),
])
def test_sparse_ggt_shapes(env, d, m, k, eps, T, kw):
    torch, oracle_mod, binding = env
    w = run_parity(torch, oracle_mod, binding, d, m, k, eps, _edge_grads(d, T, d + m), ggt=True, **kw)
    print((d, m, k), kw, w)


def test_sparse_ggt_duplicate_rows_checkpoint_and_limits(env):
    """Identical gradients with k = d make G^T G singular (pseudo-inverse path); export/import
    rebuilds the decomposition that apply replays; m > 128 is refused."""
    torch, oracle_mod, binding = env
    d, m, eps = 6_000, 5, 1e-2
    rng = np.random.default_rng(31)
    g0 = rng.standard_normal(d).astype(np.float32)
    grads = [g0, g0, rng.standard_normal(d).astype(np.float32), g0]
    w = run_parity(torch, oracle_mod, binding, d, m, d, eps, iter(grads), ggt=True, apply_every=1)
    print("ggt duplicates", w)
    dev = torch.device("cuda:0")
    a = binding.Efcp(d, m, 60, eps, ggt=True)
    b = binding.Efcp(d, m, 60, eps, ggt=True)
    c = binding.Efcp(d, m, 60, eps)
    try:
        out_a, out_b = torch.empty(d, device=dev), torch.empty(d, device=dev)
        gs = [torch.from_numpy(g).to(dev) for g in _edge_grads(d, 8, 5)]
        for g in gs[:5]:
            a.step(g, out_a)
        blob = a.export_state()
        with pytest.raises(binding.EfcpError):
            c.import_state(blob)
        b.import_state(blob)
        x = gs[7]
        a.apply(x, out_a)
        b.apply(x, out_b)
        torch.cuda.synchronize()
        assert torch.equal(out_a, out_b)
        for g in gs[5:]:
            a.step(g, out_a)
            b.step(g, out_b)
            torch.cuda.synchronize()
            assert torch.equal(out_a, out_b)
        with pytest.raises(binding.EfcpError):
            binding.Efcp(d, 129, 60, eps, ggt=True)
    finally:
        a.destroy(); b.destroy(); c.destroy()


# ---------------------------------------------------------------------------
# HIP graphs: the entry points enqueue kernels only (no allocation, no host
# synchronisation, no memset nodes), so a caller may capture them

def test_step_and_apply_under_hip_graph_capture(env):
    """A step captured into a graph and launched once equals the eager step of a twin
    context; efcp_apply captured once and replayed with new x contents equals
    the eager call every time (eager work and synchronisations in between)."""
    torch, _, binding = env
    dev = torch.device("cuda:0")
    d, m, k, lam = 200_003, 4, 1500, 1e-3
    for values in (binding.VALUES_FP32, binding.VALUES_BF16):
        a = binding.Efcp(d, m, k, lam, values=values)
        b = binding.Efcp(d, m, k, lam, values=values)
        try:
            s = torch.cuda.Stream()
            gen = torch.Generator(device=dev)
            gen.manual_seed(7)
            g = torch.empty(d, device=dev)
            oa, ob = torch.empty(d, device=dev), torch.empty(d, device=dev)
            for t in range(m + 3):                       # past the point where steps evict
                g.normal_(generator=gen)
                torch.cuda.synchronize()                 # g is written on torch's stream, read on s
                a.step(g, oa, stream=s)
                b.step(g, ob, stream=s)
                s.synchronize()
            assert torch.equal(oa, ob)
            for rep in range(3):                         # b's next steps: one fresh graph each
                g.normal_(generator=gen)
                torch.cuda.synchronize()
                a.step(g, oa, stream=s)
                s.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=s):
                    b.step(g, ob, stream=s)
                ob.zero_()
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                assert torch.equal(oa, ob), f"captured step {rep} differs from the eager one"
                assert np.array_equal(bits(a.get_error()), bits(b.get_error()))
            x = torch.empty(d, device=dev)
            y, y_ref = torch.empty(d, device=dev), torch.empty(d, device=dev)
            x.normal_(generator=gen)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=s):
                a.apply(x, y, stream=s)
            for rep in range(4):
                x.normal_(generator=gen)                 # new contents, same buffer
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                a.apply(x, y_ref, stream=s)
                s.synchronize()
                assert torch.equal(y, y_ref), f"replay {rep} of the captured apply differs"
        finally:
            a.destroy()
            b.destroy()


def test_two_contexts_on_two_streams_do_not_share_state(env):
    """Two contexts of different shapes (and slice widths) stepping at the same time on two streams,
    no synchronisation in between: each must leave exactly what a twin leaves that ran alone.
    (Nothing in the library is process-wide except the scratch array of efcp_apply_noalloc.)"""
    torch, _, binding = env
    dev = torch.device("cuda:0")
    shapes = [dict(d=180_001, m=7, k=1_500, lam=1e-3), dict(d=50_000, m=4, k=900, lam=1e-2, slice_width=512)]
    T = 14
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    grads = [[torch.randn(sh["d"], device=dev, generator=gen) * torch.exp(torch.randn(sh["d"], device=dev, generator=gen))
              for _ in range(T)] for sh in shapes]
    torch.cuda.synchronize()

    def run(concurrent):
        ctxs = [binding.Efcp(sh["d"], sh["m"], sh["k"], sh["lam"], slice_width=sh.get("slice_width", 0)) for sh in shapes]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        outs = [[torch.empty(sh["d"], device=dev) for _ in range(T)] for sh in shapes]
        if concurrent:
            for t in range(T):
                for i in (0, 1):
                    ctxs[i].step(grads[i][t], outs[i][t], stream=streams[i])
        else:
            for i in (0, 1):
                for t in range(T):
                    ctxs[i].step(grads[i][t], outs[i][t], stream=streams[i])
                streams[i].synchronize()
        torch.cuda.synchronize()
        res = [(torch.stack(outs[i]).cpu().numpy(), ctxs[i].get_error(), ctxs[i].get_small()) for i in (0, 1)]
        for c in ctxs:
            c.destroy()
        return res
    alone, together = run(False), run(True)
    for (oa, ea, sa), (ob, eb, sb) in zip(alone, together):
        assert np.array_equal(bits(oa), bits(ob))
        assert np.array_equal(bits(ea), bits(eb))
        assert sa["step"] == sb["step"] == T and np.array_equal(sa["S"], sb["S"]) and np.array_equal(sa["coef"], sb["coef"])


@pytest.mark.parametrize("topk_block", [16_384, 0])
def test_single_stream_option_gives_the_same_bits(env, topk_block):
    """efcp_options.single_stream = 1 runs the eviction update on the caller's stream instead
    of the library's second stream: same kernels, other order of launches, identical results
    through the fill of the window and on into evicting steps.  It decides something with Top-k
    in blocks only (with the global Top-k the update is part of a selection kernel and the two
    contexts enqueue the same launches)."""
    torch, _, binding = env
    d, m, lam = 90_001, 6, 1e-3
    k = 120 if topk_block else 700
    a = binding.Efcp(d, m, k, lam, topk_block=topk_block)
    b = binding.Efcp(d, m, k, lam, topk_block=topk_block, single_stream=True)
    s = synth.GradientStream(d, 0.9, 8)
    g = torch.empty(d, dtype=torch.float32, device="cuda:0")
    oa, ob = torch.empty_like(g), torch.empty_like(g)
    for t in range(1, m + 9):
        g.copy_(torch.from_numpy(s.next()))
        a.step(g, oa)
        b.step(g, ob)
        torch.cuda.synchronize()
        assert torch.equal(oa, ob), f"step {t}"
        sa, sb = a.get_small(), b.get_small()
        assert all(np.array_equal(sa[key], sb[key]) for key in ("S", "q", "coef"))
    assert np.array_equal(bits(a.get_error()), bits(b.get_error()))
    a.destroy()
    b.destroy()


@pytest.mark.parametrize("kw", [dict(), dict(values=1), dict(topk_block=16_384, k=40),
                                dict(compressed=True), dict(update=True), dict(ggt=True, values=1)])
def test_one_captured_step_replays_as_every_later_step(env, kw):
    """No kernel argument of a step depends on the step number (slot, rows filled and whether a
    row is evicted are read from device memory, which the step itself advances), so ONE HIP
    graph captured from the very first step of a context is every later step as well: replayed
    m + 7 times with new gradient contents in the captured buffer -- through the fill of the
    window and on into steps that evict -- it must leave bit for bit what the same number of
    eager efcp_step calls leave in a twin context: output (or updated parameters), every stored
    row, e, S, q, coef, the step count.  Eager work and synchronisations sit between replays."""
    torch, _, binding = env
    dev = torch.device("cuda:0")
    kw = dict(kw)
    compressed, update = kw.pop("compressed", False), kw.pop("update", False)
    d, m, lam = 150_011, 5, 1e-3
    k = kw.pop("k", 1200)
    a = binding.Efcp(d, m, k, lam, **kw)
    b = binding.Efcp(d, m, k, lam, **kw)
    xs = binding.X_COMPRESSED if compressed else binding.X_GRAD
    try:
        s = torch.cuda.Stream()
        gen = torch.Generator(device=dev)
        gen.manual_seed(3)
        scale = torch.exp(torch.randn(d, device=dev, generator=gen))
        g = torch.empty(d, device=dev)
        oa, ob = torch.zeros(d, device=dev), torch.zeros(d, device=dev)

        def call(ctx, out):
            if update:
                ctx.step_ex(g, xs, param=out, lr=1e-4, weight_decay=0.1, stream=s)
            else:
                ctx.step_ex(g, xs, out=out, stream=s)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):          # recorded, not run: b is still at step 0
            call(b, ob)
        assert b.get_small()["step"] == 0
        for t in range(1, m + 8):
            g.normal_(generator=gen)
            g.mul_(scale)
            torch.cuda.synchronize()
            call(a, oa)
            s.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(oa, ob), f"replay {t} differs from eager step {t}"
            sa, sb = a.get_small(), b.get_small()
            assert sa["step"] == sb["step"] == t
            for key in ("S", "q", "coef"):
                assert np.array_equal(sa[key], sb[key]), f"replay {t}: {key} differs"
            slot = (t - 1) % m
            (ia, va), (ib, vb) = a.get_row(slot), b.get_row(slot)
            assert np.array_equal(ia, ib) and np.array_equal(bits(va), bits(vb))
            assert np.array_equal(bits(a.get_error()), bits(b.get_error()))
        # the context that only ever replayed its graph goes on eagerly, still in step with its twin
        g.normal_(generator=gen)
        torch.cuda.synchronize()
        call(a, oa)
        call(b, ob)
        s.synchronize()
        assert torch.equal(oa, ob) and b.get_small()["step"] == m + 8
    finally:
        a.destroy()
        b.destroy()


@pytest.mark.parametrize("bf16", [False, True])
def test_caller_workspace_full_of_nan_patterns(env, bf16):
    """The library must not depend on what a workspace held before: entries outside
    a run (the unused tail of a row's last group, rows not inserted yet) are multiplied
    by zero in the SP pass, so they have to be finite from the start.  Here the caller's
    workspace is all 0xFF bytes (NaN in every format) before efcp_create."""
    torch, oracle_mod, binding = env
    dev = torch.device("cuda:0")
    d, m, k, lam = 20_001, 8, 201, 1e-3                  # k is not a multiple of the group size
    values = binding.VALUES_BF16 if bf16 else binding.VALUES_FP32
    nbytes = binding.efcp_workspace_bytes(d, m, k, values)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=dev)
    ctx = binding.Efcp(d, m, k, lam, workspace=ws, values=values)
    o = oracle_mod.Oracle(d, m, k, lam, values_bf16=bf16)
    try:
        g_d = torch.empty(d, device=dev)
        out_d = torch.empty(d, device=dev)
        for t, g in enumerate(_edge_grads(d, 12, 3), 1):
            y = o.step(g)
            g_d.copy_(torch.from_numpy(g))
            ctx.step(g_d, out_d)
            torch.cuda.synchronize()
            out = out_d.cpu().numpy()
            assert np.isfinite(out).all()
            assert rel_l2(out, y) <= 1e-3, f"step {t}"
            assert np.array_equal(bits(ctx.get_error()), bits(o.error))
    finally:
        ctx.destroy()
        o.close()
