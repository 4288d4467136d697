"""Pins for the oracle's error feedback and Top-k (Algorithm 1, lines 5-7;
Top-k sparsification of Section "Compressing Preconditioners via Sparsity").

Nothing here re-types the oracle's sort: the selection is pinned by brute
force (repeated arg-max), by numpy's stable sort, by closed-form cases and by
the order property that defines a correct Top-k.  The error feedback is pinned
by the telescoping identity sum_t c_t + xi_T = sum_t g_t, made bit-exact with
small-integer gradients.
"""
import numpy as np
import pytest

from paper_2306_06098_amd import synth


def _key(a):
    return a.view(np.uint32) & np.uint32(0x7FFFFFFF)


def _brute_topk(a, k):
    """Repeated arg-max of the magnitude key; np.argmax returns the first
    (lowest-index) maximum, which is the tie rule."""
    key = _key(a).astype(np.int64)
    chosen = []
    for _ in range(k):
        j = int(np.argmax(key))
        chosen.append(j)
        key[j] = -1
    return np.sort(np.array(chosen, dtype=np.int32))


@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force_tiny(oracle_mod, seed):
    rng = np.random.default_rng(seed)
    d = int(rng.integers(1, 65))
    k = int(rng.integers(1, d + 1))
    # few distinct magnitudes -> many ties, both signs, signed zeros
    a = rng.integers(-3, 4, size=d).astype(np.float32)
    a[rng.random(d) < 0.2] *= np.float32(-0.0) if seed % 2 else np.float32(1.0)
    idx, val = oracle_mod.topk(a, k)
    assert np.array_equal(idx, _brute_topk(a, k))
    assert np.array_equal(val.view(np.uint32), a[idx].view(np.uint32))


def test_topk_stable_sort_1e6(oracle_mod):
    rng = np.random.default_rng(11)
    d, k = 1_000_003, 10_007
    a = (rng.standard_normal(d) * np.exp(rng.standard_normal(d))).astype(np.float32)
    a = np.round(a * 64) / 64            # quantise: forces ties at the threshold
    a = a.astype(np.float32)
    order = np.argsort(-(_key(a).astype(np.int64)), kind="stable")
    expect = np.sort(order[:k]).astype(np.int32)
    idx, val = oracle_mod.topk(a, k)
    assert np.array_equal(idx, expect)
    assert np.array_equal(val.view(np.uint32), a[idx].view(np.uint32))
    # the defining order property
    key = _key(a)
    sel = np.zeros(d, bool)
    sel[idx] = True
    tau = key[sel].min()
    assert key[~sel].max() <= tau
    ties = np.nonzero(key == tau)[0]
    n_sel_ties = int(sel[ties].sum())
    assert sel[ties[:n_sel_ties]].all() and not sel[ties[n_sel_ties:]].any()


def test_topk_closed_forms(oracle_mod):
    d, k = 1000, 37
    for fill in (np.float32(2.5), np.float32(0.0), np.float32(-0.0)):
        a = np.full(d, fill, dtype=np.float32)
        idx, val = oracle_mod.topk(a, k)
        assert np.array_equal(idx, np.arange(k, dtype=np.int32))      # all equal -> first k
        assert np.array_equal(val.view(np.uint32), a[:k].view(np.uint32))
    a = np.zeros(d, np.float32)
    a[::2] = -0.0                                     # +0 and -0 tie
    idx, _ = oracle_mod.topk(a, k)
    assert np.array_equal(idx, np.arange(k, dtype=np.int32))
    a = np.arange(d, dtype=np.float32) * np.where(np.arange(d) % 2, -1, 1).astype(np.float32)
    idx, val = oracle_mod.topk(a, k)
    assert np.array_equal(idx, np.arange(d - k, d, dtype=np.int32))    # magnitude, not signed value
    assert np.array_equal(val, a[d - k:])
    idx, _ = oracle_mod.topk(a, 1)
    assert idx[0] == d - 1
    idx, val = oracle_mod.topk(a, d)
    assert np.array_equal(idx, np.arange(d, dtype=np.int32)) and np.array_equal(val, a)


def test_topk_extreme_values(oracle_mod):
    tiny = np.float32(1e-45)               # smallest subnormal
    a = np.array([0.0, tiny, -tiny, 3.0e38, -3.4e38, 1.0, -1.0, 2 * tiny], dtype=np.float32)
    idx, val = oracle_mod.topk(a, 3)
    assert list(idx) == [3, 4, 5]           # 1.0 ties with -1.0 -> lower index
    idx, _ = oracle_mod.topk(a, 6)
    assert list(idx) == [1, 3, 4, 5, 6, 7]   # subnormals ordered, not flushed


def test_ef_telescoping_exact_with_integer_gradients(oracle_mod):
    """sum_t c_t + xi_T == sum_t g_t exactly: all values are small integers,
    so every fp32 operation is exact and the identity must hold bit for bit."""
    d, m, k, T = 4096, 5, 41, 23
    o = oracle_mod.Oracle(d, m, k, 1e-2)
    stream = synth.integer_stream(d, seed=5)
    sum_g = np.zeros(d, np.float64)
    sum_c = np.zeros(d, np.float64)
    e_prev = np.zeros(d, np.float32)
    for t in range(1, T + 1):
        g = next(stream)
        o.step(g)
        idx, val = o.row(o.newest_slot)
        a = e_prev + g                              # exact
        assert np.array_equal(val, a[idx])          # stored values are a at the indices
        e = o.error
        assert not e[idx].any() and not np.signbit(e[idx]).any()     # +0 where selected
        mask = np.ones(d, bool)
        mask[idx] = False
        assert np.array_equal(e[mask], a[mask])     # untouched elsewhere
        assert len(np.unique(idx)) == k and (np.diff(idx) > 0).all()
        sum_g += g
        sum_c[idx] += val
        assert np.array_equal(sum_c + e, sum_g)
        e_prev = e.copy()


def test_ef_telescoping_float(oracle_mod):
    wl = synth.WORKLOADS["tiny"]
    o = oracle_mod.Oracle(wl.d, wl.m, wl.k, wl.lam)
    s = synth.GradientStream(wl.d, wl.rho, wl.seed)
    sum_g = np.zeros(wl.d)
    sum_c = np.zeros(wl.d)
    for _ in range(40):
        g = s.next()
        o.step(g)
        idx, val = o.row(o.newest_slot)
        sum_g += g
        sum_c[idx] += val
    resid = np.linalg.norm(sum_c + o.error - sum_g) / np.linalg.norm(sum_g)
    assert resid < 40 * 1e-7


def test_ef_k_equals_d_keeps_error_zero(oracle_mod):
    d = 300
    o = oracle_mod.Oracle(d, 3, d, 1e-1)
    rng = np.random.default_rng(2)
    for _ in range(5):
        g = rng.standard_normal(d).astype(np.float32)
        o.step(g)
        assert not o.error.any()
        idx, val = o.row(o.newest_slot)
        assert np.array_equal(idx, np.arange(d)) and np.array_equal(val, g)


def test_ring_slot_order_and_eviction(oracle_mod):
    """Slot (t-1) mod m is written at step t and the oldest row is replaced."""
    d, m, k = 512, 4, 9
    o = oracle_mod.Oracle(d, m, k, 1e-2)
    rng = np.random.default_rng(3)
    history = []
    for t in range(1, 11):
        g = rng.standard_normal(d).astype(np.float32)
        o.step(g)
        assert o.newest_slot == (t - 1) % m and o.filled == min(t, m)
        history.append(tuple(x.copy() for x in o.row(o.newest_slot)))
        for back in range(min(t, m)):               # last m rows are all still there
            slot = (t - 1 - back) % m
            i, v = o.row(slot)
            assert np.array_equal(i, history[t - 1 - back][0])
            assert np.array_equal(v, history[t - 1 - back][1])


# ---------------------------------------------------------------------------
# bfloat16 window values (Section "Format for V")

def test_bf16_rounding_matches_torch_bfloat16(oracle_mod):
    """The oracle's fp32 -> bf16 rounding against torch's CPU conversion
    (round to nearest even), on random values, exact ties and the extremes."""
    import torch
    rng = np.random.default_rng(5)
    vals = (rng.standard_normal(4000) * np.exp(rng.uniform(-60, 60, 4000))).astype(np.float32)
    ties = np.array([0x3F808000, 0x3F818000, 0x3F80FFFF, 0x3F808001, 0x00008000, 0x00018000,
                     0x7F7F7FFF, 0xBF808000, 0x80000000, 0x00000000], dtype=np.uint32).view(np.float32)
    allv = np.concatenate([vals, ties])
    ref = torch.from_numpy(allv).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle_mod.bf16_round(float(v)) for v in allv], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    assert not (got.view(np.uint32) & np.uint32(0xFFFF)).any()


def test_bf16_window_error_feedback_keeps_the_rounding_remainder(oracle_mod):
    """xi = a - c with c = bf16(a) on the selection: the remainder stays in e,
    so the telescoping identity still holds exactly (integer gradients)."""
    d, m, k, T = 3000, 4, 60, 25
    o = oracle_mod.Oracle(d, m, k, 1e-2, values_bf16=True)
    stream = synth.integer_stream(d, seed=6, lo=-300, hi=300)      # beyond bf16's 8 exact bits
    sum_g = np.zeros(d)
    sum_c = np.zeros(d)
    e_prev = np.zeros(d, np.float32)
    saw_remainder = False
    for _ in range(T):
        g = next(stream)
        o.step(g)
        idx, val = o.row(o.newest_slot)
        a = e_prev + g
        assert not (val.view(np.uint32) & np.uint32(0xFFFF)).any()          # representable in bf16
        assert (np.abs(val - a[idx]) <= np.abs(a[idx]) * 2.0 ** -8).all()   # half an ulp of 8 bits
        e = o.error
        assert np.array_equal(e[idx], a[idx] - val)
        saw_remainder |= bool(e[idx].any())
        mask = np.ones(d, bool); mask[idx] = False
        assert np.array_equal(e[mask], a[mask])
        # selection is by |a| in fp32, before rounding
        assert np.array_equal(idx, oracle_mod.topk(a, k)[0])
        sum_g += g
        sum_c[idx] += val
        assert np.array_equal(sum_c + e, sum_g)
        e_prev = e.copy()
    assert saw_remainder


# ---------------------------------------------------------------------------
# Top-k applied in blocks (Section "Sparsity Pattern")

def test_blockwise_topk_keeps_exactly_kb_per_block(oracle_mod):
    """Every full block holds exactly kb selected entries, and they are that
    block's own Top-kb by brute force; the ragged last block keeps the same
    share rounded up; e = a - c and the telescoping identity still hold."""
    d, m, B, kb, T = 1000, 3, 128, 7, 9                 # 7 full blocks + a tail of 104
    o = oracle_mod.Oracle(d, m, kb, 1e-2, block=B)
    tail_keep = -(-kb * (d % B) // B)
    assert o.k == (d // B) * kb + tail_keep == 55
    stream = synth.integer_stream(d, seed=12)            # many ties
    e_prev = np.zeros(d, np.float32)
    sum_g = np.zeros(d)
    sum_c = np.zeros(d)
    for _ in range(T):
        g = next(stream)
        o.step(g)
        a = e_prev + g
        idx, val = o.row(o.newest_slot)
        assert (np.diff(idx) > 0).all()
        expect = []
        for lo in range(0, d, B):
            blk = a[lo:lo + B]
            keep = kb if blk.size == B else tail_keep
            in_blk = idx[(idx >= lo) & (idx < lo + B)]
            assert in_blk.size == keep
            expect.append(_brute_topk(blk, keep) + lo)
        assert np.array_equal(idx, np.concatenate(expect))
        assert np.array_equal(val, a[idx])
        e = o.error
        assert not e[idx].any()
        mask = np.ones(d, bool); mask[idx] = False
        assert np.array_equal(e[mask], a[mask])
        sum_g += g
        sum_c[idx] += val
        assert np.array_equal(sum_c + e, sum_g)
        e_prev = e.copy()


def test_blockwise_with_one_block_is_global_topk(oracle_mod):
    d, k = 777, 31
    a = oracle_mod.Oracle(d, 4, k, 1e-2, block=d)         # a single block covering everything
    b = oracle_mod.Oracle(d, 4, k, 1e-2)
    c = oracle_mod.Oracle(d, 4, k, 1e-2, block=4 * d)     # block larger than d: only a "tail"
    assert a.k == k and c.k == -(-k * d // (4 * d))
    rng = np.random.default_rng(14)
    for _ in range(6):
        g = rng.standard_normal(d).astype(np.float32)
        ya, yb = a.step(g), b.step(g)
        assert np.array_equal(a.row(a.newest_slot)[0], b.row(b.newest_slot)[0])
        assert np.array_equal(a.error, b.error) and np.array_equal(ya, yb)


def test_blockwise_differs_from_global_when_mass_is_concentrated(oracle_mod):
    """All large entries in one block: global Top-k takes them all, blockwise
    may take only kb of them -- the rest stays in the error feedback."""
    d, B, kb = 512, 128, 4
    g = np.full(d, 0.5, np.float32)
    g[:16] = np.arange(16, 0, -1, dtype=np.float32) + 10
    o = oracle_mod.Oracle(d, 2, kb, 1e-2, block=B)
    o.step(g)
    idx, _ = o.row(0)
    assert list(idx[:kb]) == [0, 1, 2, 3]
    assert np.array_equal(idx[kb:], np.concatenate([np.arange(B * b, B * b + kb) for b in (1, 2, 3)]))
    assert np.array_equal(o.error[4:16], g[4:16])


def test_topk_property_search(oracle_mod):
    """hypothesis searches for a vector on which eo_topk is not the k largest magnitudes with ties
    to the lower index: the selected set must be exactly what repeated arg-max picks, whatever
    mix of ties, signed zeros, subnormals, huge values and lengths it comes up with."""
    hypothesis = pytest.importorskip("hypothesis")
    from hypothesis import given, settings, strategies as st
    pool = [0.0, -0.0, 1.0, -1.0, 1.5, -1.5, 2.0, 1e-45, -1e-45, 1e-38, 3e38, -3e38, 0.1, -0.1, 7.0]
    vec = st.lists(st.one_of(st.sampled_from(pool), st.floats(width=32, allow_nan=False, allow_infinity=False)),
                   min_size=1, max_size=96)

    @settings(max_examples=300, deadline=None)
    @given(vec, st.data())
    def check(values, data):
        a = np.array(values, dtype=np.float32)
        k = data.draw(st.integers(1, a.size))
        idx, val = oracle_mod.topk(a, k)
        assert np.array_equal(idx, _brute_topk(a, k))
        assert np.array_equal(val.view(np.uint32), a[idx].view(np.uint32))
        key = _key(a)
        rest = np.setdiff1d(np.arange(a.size), idx)
        if rest.size:
            assert key[idx].min() >= key[rest].max()
    check()
