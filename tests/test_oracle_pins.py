"""Pins for the CPU oracle: closed forms, invariants, library cross-checks and
exhaustive enumeration on tiny cases.  No GPU, no HIP library.

Each test is chosen so that a plausible mistake in the oracle (dropped term,
wrong sign, transposed operand, off-by-one index, wrong tie rule) fails it.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import eh_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- entropy/lse
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "entropy_closed_form.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            V, n, a, H, lse = line.split()
            rows.append((int(V), int(n), float(a), float(H), float(lse)))
    return rows


@pytest.mark.parametrize("V,n,a,H_ref,lse_ref", _golden_rows())
def test_two_level_logits_closed_form(V, n, a, H_ref, lse_ref):
    # Section 3.4.1: entropy of the predicted distribution; closed form fixture.
    rng = np.random.default_rng(V + n)
    z = np.zeros(V)
    pos = rng.choice(V, size=n, replace=False)
    z[pos] = a
    H, lse, am, gap = O.softmax_stats(z)
    assert H[0] == pytest.approx(H_ref, rel=1e-11, abs=1e-15)
    assert lse[0] == pytest.approx(lse_ref, rel=1e-13)
    if a > 0:
        assert am[0] == pos.min()
        assert gap[0] == pytest.approx(0.0 if n > 1 else a)


def test_uniform_logits_give_log_V():
    V = 50304
    for c in (0.0, -3.25, 1e4):
        H, lse, am, gap = O.softmax_stats(np.full(V, c))
        # the shift costs |c| * 2**-53 of absolute accuracy in z - lse
        assert H[0] == pytest.approx(math.log(V), rel=1e-13, abs=max(1.0, abs(c)) * 4e-15)
        assert lse[0] == pytest.approx(c + math.log(V), rel=1e-13)
        assert am[0] == 0 and gap[0] == 0.0
    assert math.log(V) == pytest.approx(10.825839875788878, rel=1e-15)


def test_dominant_logit_entropy_goes_to_zero():
    V = 50304
    prev = None
    for a in (20.0, 30.0, 40.0, 80.0, 800.0):
        z = np.zeros(V)
        z[V - 1] = a
        H, lse, am, _ = O.softmax_stats(z)
        assert 0.0 <= H[0] < 3e-3
        assert prev is None or H[0] <= prev
        assert am[0] == V - 1
        prev = H[0]
    assert prev == 0.0  # exp underflow gives exactly 0 log 0 = 0


def test_shift_permutation_invariance_and_bounds():
    rng = np.random.default_rng(7)
    V = 4099
    for scale in (0.5, 2.0, 8.0):
        z = rng.normal(size=V) * scale
        H, lse, am, gap = O.softmax_stats(z)
        assert 0.0 <= H[0] <= math.log(V)
        assert z.max() <= lse[0] <= z.max() + math.log(V)
        for c in (1.0, -1.0, 100.0, -100.0, 1e4, -1e4):
            H2, lse2, am2, gap2 = O.softmax_stats(z + c)
            assert H2[0] == pytest.approx(H[0], abs=1e-9)
            assert lse2[0] == pytest.approx(lse[0] + c, rel=1e-12)
            assert am2[0] == am[0]
        perm = rng.permutation(V)
        H3, lse3, am3, gap3 = O.softmax_stats(z[perm])
        assert H3[0] == pytest.approx(H[0], rel=1e-12)
        assert lse3[0] == pytest.approx(lse[0], rel=1e-13)
        assert perm[am3[0]] == am[0]
        assert gap3[0] == pytest.approx(gap[0])


def test_softmax_stats_against_scipy():
    # special case reducing to library routines
    from scipy.special import logsumexp, softmax
    from scipy.stats import entropy
    rng = np.random.default_rng(11)
    z = rng.normal(size=(5, 1000)) * np.array([0.3, 1, 3, 9, 27])[:, None]
    H, lse, am, gap = O.softmax_stats(z)
    np.testing.assert_allclose(lse, logsumexp(z, axis=1), rtol=1e-13)
    np.testing.assert_allclose(H, entropy(softmax(z, axis=1), axis=1), rtol=1e-10, atol=1e-14)
    np.testing.assert_array_equal(am, z.argmax(axis=1))
    srt = np.sort(z, axis=1)
    np.testing.assert_allclose(gap, srt[:, -1] - srt[:, -2])


def test_exhaustive_V8_three_level_logits():
    # brute force: all 3^8 logit vectors over {0,1,2}; naive formulas in pure Python
    V = 8
    allz = np.array(list(itertools.product((0.0, 1.0, 2.0), repeat=V)))
    H, lse, am, gap = O.softmax_stats(allz)
    for r, z in enumerate(allz):
        e = [math.exp(v) for v in z]
        Z = sum(e)
        p = [v / Z for v in e]
        Hn = -sum(q * math.log(q) for q in p)
        assert H[r] == pytest.approx(Hn, rel=1e-12)
        assert lse[r] == pytest.approx(math.log(Z), rel=1e-13)
        best = max(z)
        assert am[r] == list(z).index(best)          # lowest index on ties
        second = sorted(z)[-2]
        assert gap[r] == best - second


def test_nan_row_gives_nan():
    z = np.zeros((2, 16))
    z[1, 3] = np.nan
    H, lse, am, gap = O.softmax_stats(z)
    assert np.isfinite(H[0]) and np.isnan(H[1]) and np.isnan(lse[1])


# ------------------------------------------------------------------ LayerNorm
def test_layernorm_constant_row_gives_beta():
    d = 64
    rng = np.random.default_rng(0)
    g, b = rng.normal(size=d), rng.normal(size=d)
    y = O.layernorm(np.full((3, d), 4.75), g, b)
    np.testing.assert_array_equal(y, np.broadcast_to(b, (3, d)))


def test_layernorm_moments_and_scale_invariance():
    rng = np.random.default_rng(1)
    d, eps = 512, 1e-5
    h = rng.normal(size=(4, d)) * np.array([0.1, 1.0, 7.0, 300.0])[:, None] + 3.0
    one, zero = np.ones(d), np.zeros(d)
    xh = O.layernorm(h, one, zero, eps)
    var = h.var(axis=1)                       # numpy's biased variance
    np.testing.assert_allclose(xh.mean(axis=1), 0.0, atol=1e-13)
    np.testing.assert_allclose((xh ** 2).mean(axis=1), var / (var + eps), rtol=1e-12)
    a = O.layernorm(h, one, zero, 0.0)
    b = O.layernorm(5.5 * h - 17.0, one, zero, 0.0)
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-11)
    c = O.layernorm(-2.0 * h, one, zero, 0.0)
    np.testing.assert_allclose(c, -a, rtol=1e-9, atol=1e-11)  # sign is kept


def test_layernorm_d2_closed_form_and_affine():
    u, v, eps = 3.0, -1.5, 1e-5
    g = np.array([2.0, -3.0])
    b = np.array([0.25, 0.5])
    y = O.layernorm(np.array([[u, v]]), g, b, eps)[0]
    s = abs(u - v) / math.sqrt((u - v) ** 2 + 4 * eps)
    assert y[0] == pytest.approx(g[0] * s + b[0], rel=1e-14)
    assert y[1] == pytest.approx(-g[1] * s + b[1], rel=1e-14)


def test_layernorm_against_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    d = 160
    h = rng.normal(size=(6, d)) * 3 + 1
    g, b = rng.normal(size=d), rng.normal(size=d)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(h), (d,), torch.from_numpy(g),
                                         torch.from_numpy(b), eps=1e-5).numpy()
    np.testing.assert_allclose(O.layernorm(h, g, b, 1e-5), ref, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ projection
def test_projection_selector_rows():
    # W row i = c_i * e_{j(i)}  ->  z_i = c_i * y_{j(i)}; catches a transposed operand
    rng = np.random.default_rng(3)
    d, V = 12, 40
    y = rng.normal(size=(5, d))
    j = rng.integers(0, d, size=V)
    c = rng.normal(size=V)
    W = np.zeros((V, d))
    W[np.arange(V), j] = c
    z = O.head_logits(y, W)
    np.testing.assert_allclose(z, y[:, j] * c, rtol=1e-15)
    bias = rng.normal(size=V)
    np.testing.assert_allclose(O.head_logits(y, W, bias), y[:, j] * c + bias, rtol=1e-15)


def test_projection_identity_block():
    d, V = 8, 20
    W = np.zeros((V, d))
    W[:d] = np.eye(d)
    y = np.arange(1.0, 2 * d + 1).reshape(2, d)
    z = O.head_logits(y, W)
    np.testing.assert_array_equal(z[:, :d], y)
    np.testing.assert_array_equal(z[:, d:], 0.0)


def test_head_eval_against_torch_pipeline():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(4)
    d, V, R = 96, 777, 9
    h = rng.normal(size=(R, d)) * rng.uniform(0.5, 8, size=(R, 1))
    g = 1 + 0.02 * rng.normal(size=d)
    b = 0.02 * rng.normal(size=d)
    W = rng.normal(size=(V, d)) * 3 / math.sqrt(d)
    H, lse, am, gap = O.head_eval(h, g, b, W)
    th = torch.from_numpy
    y = torch.nn.functional.layer_norm(th(h), (d,), th(g), th(b), eps=1e-5)
    z = torch.nn.functional.linear(y, th(W))
    lp = torch.log_softmax(z, dim=-1)
    ent = torch.distributions.Categorical(logits=z).entropy()
    np.testing.assert_allclose(H, ent.numpy(), rtol=1e-10)
    np.testing.assert_allclose(lse, torch.logsumexp(z, -1).numpy(), rtol=1e-12)
    np.testing.assert_array_equal(am, lp.argmax(-1).numpy())


# ------------------------------------------------------------------ bf16
def test_bf16_roundtrip_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    v = O.bf16_bits_to_f64(bits)
    fin = np.isfinite(v)
    r = O.round_to_bf16(v)
    np.testing.assert_array_equal(r[fin], v[fin])
    np.testing.assert_array_equal(O.f64_to_bf16_bits(v[fin]), bits[fin])


def test_bf16_ties_to_even_and_neighbours():
    bits = np.arange(0x0001, 0x7F7F, dtype=np.uint32).astype(np.uint16)  # positive finite, incl. subnormals
    lo = O.bf16_bits_to_f64(bits)
    hi = O.bf16_bits_to_f64(bits + np.uint16(1))
    mid = (lo + hi) / 2                      # exact in fp64
    even = np.where(bits % 2 == 0, lo, hi)
    np.testing.assert_array_equal(O.round_to_bf16(mid), even)
    np.testing.assert_array_equal(O.round_to_bf16(-mid), -even)
    np.testing.assert_array_equal(O.round_to_bf16(np.nextafter(mid, np.inf)), hi)
    np.testing.assert_array_equal(O.round_to_bf16(np.nextafter(mid, -np.inf)), lo)


def test_bf16_hand_picked():
    f = O.round_to_bf16
    assert f(np.array([1.0 + 2.0 ** -8]))[0] == 1.0              # tie -> even (1.0)
    assert f(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6  # tie -> even (up)
    assert f(np.array([1.00390625 + 1e-9]))[0] == 1.0078125
    big = O.bf16_bits_to_f64(np.array([0x7F7F], dtype=np.uint16))[0]   # largest finite
    assert f(np.array([big]))[0] == big
    assert np.isinf(f(np.array([big * (1 + 2.0 ** -8)]))[0])      # tie at the top rounds to inf
    assert f(np.array([big * (1 + 2.0 ** -9)]))[0] == big
    tiny = 2.0 ** -133                                            # smallest subnormal
    assert f(np.array([tiny * 0.5]))[0] == 0.0                    # tie -> even (0)
    assert f(np.array([tiny * 0.75]))[0] == tiny
    z = f(np.array([0.0, -0.0, np.inf, -np.inf, np.nan]))
    assert z[0] == 0.0 and np.signbit(z[1]) and np.isinf(z[2]) and np.isinf(z[3]) and np.isnan(z[4])


def test_bf16_against_torch_rne():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    x = (rng.normal(size=200000) * np.exp(rng.uniform(-60, 60, size=200000))).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_to_bf16(x.astype(np.float64)), ref)


def test_layernorm_bf16_output_is_rounded_fp64_result():
    rng = np.random.default_rng(6)
    d = 256
    h = rng.normal(size=(3, d))
    g, b = np.ones(d), np.zeros(d)
    y = O.layernorm(h, g, b, 1e-5, bf16_out=True)
    full = O.layernorm(h, g, b, 1e-5)
    np.testing.assert_array_equal(y, O.round_to_bf16(full))
    assert np.all(np.abs(y - full) <= np.abs(full) * 2.0 ** -8)
    O.f64_to_bf16_bits(y)  # raises if not representable


# ------------------------------------------------------------------ exit rule
@pytest.mark.parametrize("n_heads", [1, 2, 3, 4, 5, 6])
def test_exit_rule_all_patterns(n_heads):
    tau = np.linspace(0.5, 3.0, n_heads)
    for pattern in itertools.product((False, True), repeat=n_heads):
        H = [tau[k] - 0.1 if below else tau[k] + 0.1 for k, below in enumerate(pattern)]
        early = [k for k in range(n_heads - 1) if pattern[k]]
        expect = early[0] if early else n_heads - 1
        assert O.exit_rule(H, tau) == expect


def test_exit_rule_strict_and_nan():
    tau = [1.0, 1.0, 1.0]
    assert O.exit_rule([1.0, 1.0, 5.0], tau) == 2          # equality does not exit
    assert O.exit_rule([np.nan, 0.5, 5.0], tau) == 1       # NaN never passes
    assert O.exit_rule([np.nextafter(1.0, 0), 0.0, 0.0], tau) == 0


def test_cascade_equals_masked_full_evaluation():
    rng = np.random.default_rng(8)
    d, V, R, n_heads = 32, 200, 40, 5
    Ws = [rng.normal(size=(V, d)) * (0.5 + 1.2 * l) / math.sqrt(d) for l in range(n_heads)]
    gs = [1 + 0.02 * rng.normal(size=d) for _ in range(n_heads)]
    bs = [0.02 * rng.normal(size=d) for _ in range(n_heads)]
    hs = [rng.normal(size=(R, d)) for _ in range(n_heads)]
    full_H = np.stack([O.head_eval(hs[l], gs[l], bs[l], Ws[l])[0] for l in range(n_heads)])
    full_A = np.stack([O.head_eval(hs[l], gs[l], bs[l], Ws[l])[2] for l in range(n_heads)])
    tau = np.quantile(full_H, 0.3, axis=1)
    out = O.cascade(hs, gs, bs, Ws, tau)
    assert len(set(out["exit_layer"])) > 2   # the case exercises several exits
    for r in range(R):
        k = O.exit_rule(full_H[:, r], tau)
        assert out["exit_layer"][r] == k
        assert out["token"][r] == full_A[k, r]
        assert np.all(np.isnan(out["H"][k + 1:, r]))
        np.testing.assert_allclose(out["H"][:k + 1, r], full_H[:k + 1, r], rtol=1e-12)
    for l in range(n_heads):
        expect = [r for r in range(R) if out["exit_layer"][r] >= l]
        assert list(out["active"][l]) == expect      # stable, increasing order


# ------------------------------------------------------------------ DSSD verify
@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_accepted_prefix_exhaustive(k):
    for draft in itertools.product((0, 1), repeat=k):
        for target in itertools.product((0, 1), repeat=k + 1):
            mism = [j for j in range(k) if draft[j] != target[j]]
            first = mism[0] if mism else k
            for L in range(k + 1):
                assert O.accepted_prefix(draft, target, L) == min(first, L)


def test_dssd_verify_planted_targets():
    rng = np.random.default_rng(9)
    d, V, B, k = 24, 50, 6, 4
    W = rng.normal(size=(V, d)) / math.sqrt(d)
    g, b = np.ones(d), np.zeros(d)
    tgt = rng.integers(0, V, size=(B, k + 1))
    f = 6.0 * W[tgt] + 0.05 * rng.normal(size=(B, k + 1, d))   # aligned with row tgt
    draft = tgt[:, :k].copy()
    draft[0, 0] = (draft[0, 0] + 1) % V        # reject at once
    draft[1, 2] = (draft[1, 2] + 1) % V        # accept 2
    draft[2, 3] = (draft[2, 3] + 1) % V        # accept 3
    draft_len = np.array([k, k, k, k, 2, 0])   # rows 4, 5 truncated
    acc, nxt, target, gap = O.dssd_verify(f, draft, g, b, W, draft_len)
    np.testing.assert_array_equal(target, tgt)
    np.testing.assert_array_equal(acc, [0, 2, 3, 4, 2, 0])
    np.testing.assert_array_equal(nxt, [tgt[0, 0], tgt[1, 2], tgt[2, 3], tgt[3, 4], tgt[4, 2], tgt[5, 0]])
    acc2, _, _, _ = O.dssd_verify(f, draft, g, b, W)
    np.testing.assert_array_equal(acc2, [0, 2, 3, 4, 4, 4])


# ------------------------------------------------------------------ threshold calibration
def _calibrate_by_sorting(H, t, eps):
    """The paper's procedure step by step (Section 3.4.1): sort jointly by ascending
    confidence c = -H, take suffix proportions with running sums, pick the smallest index
    that qualifies.  Only equal to the definition when no two entropies tie."""
    H = np.asarray(H, dtype=np.float64)
    order = np.argsort(-H, kind="stable")            # ascending confidence = descending entropy
    Hs, ts = H[order], np.asarray(t)[order]
    M = len(Hs)
    suffix_correct = np.cumsum(ts[::-1])[::-1]
    for j in range(M):
        if suffix_correct[j] / (M - j) >= eps:
            return float(Hs[j]), M - j
    return -np.inf, 0


def test_calibration_worked_example():
    # entropies descending: 2.0(wrong) 1.0(wrong) 0.5(wrong) 0.5(right) 0.1(right)
    # proportions of correct from each value on: 2/5, 2/4, 2/3 (both 0.5 tied), 1/1
    H = [0.1, 0.5, 0.5, 1.0, 2.0]
    t = [1, 1, 0, 0, 0]
    assert O.calibrate_threshold(H, t, 0.0) == (2.0, 5)
    assert O.calibrate_threshold(H, t, 0.4) == (2.0, 5)
    assert O.calibrate_threshold(H, t, 0.5) == (1.0, 4)
    assert O.calibrate_threshold(H, t, 0.625) == (0.5, 3)
    assert O.calibrate_threshold(H, t, 0.75) == (0.1, 1)
    assert O.calibrate_threshold(H, t, 1.0) == (0.1, 1)


def test_calibration_degenerate_sets():
    rng = np.random.default_rng(3)
    H = rng.uniform(0.0, 5.0, size=40)
    for eps in (0.0, 0.3, 1.0):
        assert O.calibrate_threshold(H, np.ones(40, dtype=int), eps) == (float(H.max()), 40)
    assert O.calibrate_threshold(H, np.zeros(40, dtype=int), 0.0) == (float(H.max()), 40)
    for eps in (1e-9, 0.5, 1.0):
        assert O.calibrate_threshold(H, np.zeros(40, dtype=int), eps) == (-np.inf, 0)
    assert O.calibrate_threshold([], [], 0.5) == (-np.inf, 0)


def test_calibration_matches_the_sorting_procedure_without_ties():
    rng = np.random.default_rng(11)
    for trial in range(60):
        M = int(rng.integers(1, 80))
        H = rng.permutation(M).astype(np.float64) * 0.07 + 0.01        # distinct
        t = (rng.random(M) < (0.9 - 0.1 * H / H.max() * 8).clip(0.05, 0.95)).astype(int)
        for eps in (0.0, 0.25, 0.5, 0.7, 0.9, 1.0):
            assert O.calibrate_threshold(H, t, eps) == _calibrate_by_sorting(H, t, eps), (trial, eps)


def test_calibration_guarantee_minimality_monotonicity_permutation():
    rng = np.random.default_rng(5)
    for trial in range(40):
        M = int(rng.integers(2, 60))
        H = np.round(rng.uniform(0, 3, size=M), 1)                      # many ties
        t = (rng.random(M) < np.exp(-H)).astype(int)
        prev = np.inf
        for eps in (0.0, 0.2, 0.4, 0.6, 0.8, 1.0):
            tau, n = O.calibrate_threshold(H, t, eps)
            assert tau <= prev                                           # stricter level, lower threshold
            prev = tau
            if tau == -np.inf:
                assert n == 0
                assert all(t[H <= v].sum() < eps * (H <= v).sum() for v in np.unique(H))
                continue
            kept = H <= tau
            assert n == kept.sum() and t[kept].sum() >= eps * n          # the guarantee
            for v in np.unique(H[H > tau]):                              # nothing larger qualifies
                assert t[H <= v].sum() < eps * (H <= v).sum()
            perm = rng.permutation(M)
            assert O.calibrate_threshold(H[perm], t[perm], eps) == (tau, n)


def test_calibration_ties_do_not_depend_on_their_order():
    # three samples tie at 1.0: right, wrong, wrong.  Taken as a whole 1/3 of them are right.
    # An index-based suffix could start between them (after the wrong ones) and see 1/1.
    H = np.array([1.0, 1.0, 1.0, 2.0])
    for t in ([1, 0, 0, 0], [0, 1, 0, 0], [0, 0, 1, 0]):
        assert O.calibrate_threshold(H, t, 0.5) == (-np.inf, 0)
        assert O.calibrate_threshold(H, t, 1 / 3) == (1.0, 3)
        assert O.calibrate_threshold(H, t, 0.25) == (2.0, 4)


def test_calibration_ignores_nan_entropies():
    H = np.array([np.nan, 0.2, 0.9, np.nan, 0.4])
    t = np.array([1, 1, 0, 1, 1])
    assert O.calibrate_threshold(H, t, 0.6) == (0.9, 3)                   # 2 of the 3 finite ones
    assert O.calibrate_threshold(H, t, 0.7) == (0.4, 2)
    assert O.calibrate_threshold([np.nan, np.nan], [1, 1], 0.0) == (-np.inf, 0)


def test_calibration_exhaustive_small():
    from fractions import Fraction
    values = (0.25, 0.5, 0.5, 1.5, 1.5, 3.0)                             # fixed entropies with ties
    for t in itertools.product((0, 1), repeat=len(values)):
        for eps in (Fraction(0), Fraction(1, 4), Fraction(1, 2), Fraction(3, 4), Fraction(1)):
            want = (-np.inf, 0)
            for v in sorted(set(values), reverse=True):
                inside = [tj for hj, tj in zip(values, t) if hj <= v]
                if Fraction(sum(inside), len(inside)) >= eps:
                    want = (v, len(inside))
                    break
            assert O.calibrate_threshold(values, t, float(eps)) == want


def test_calibration_level_at_the_boundary():
    """Candidates that sit exactly on the level or beside it.  The proportion test is the
    quotient correct / size, correctly rounded, against epsilon (Section 3.4.1): p of q samples
    meet the level typed as the decimal p/q whichever side of p/q that decimal's double lies on,
    one sample fewer does not, and the doubles next to the level decide as their order says."""
    from fractions import Fraction
    # the double nearest 0.7 lies below 7/10, those nearest 0.01 and 0.55 lie above 1/100 and 11/20
    assert Fraction(0.7) < Fraction(7, 10) and Fraction(0.01) > Fraction(1, 100) and Fraction(0.55) > Fraction(11, 20)

    def one_value(n, c, eps):          # n samples at one entropy, c of them right: a single candidate
        return O.calibrate_threshold(np.full(n, 1.25), np.array([1] * c + [0] * (n - c)), eps)

    for eps, n, c in ((0.7, 10, 7), (0.01, 100, 1), (0.55, 20, 11), (0.02, 50, 1), (0.07, 100, 7), (0.4, 5, 2),
                      (0.3, 10, 3), (0.1, 10, 1), (0.9, 10, 9), (0.6, 5, 3), (1.0, 9, 9), (0.0, 4, 0)):
        assert one_value(n, c, eps) == (1.25, n), (eps, n, c)
        if c > 0:
            assert one_value(n, c - 1, eps) == (-np.inf, 0), (eps, n, c)
        up, down = float(np.nextafter(eps, 2.0)), float(np.nextafter(eps, -1.0))
        assert one_value(n, c, up) == (-np.inf, 0), (eps, n, c)
        if eps > 0.0:
            assert one_value(n, c, down) == (1.25, n), (eps, n, c)


def test_correctness_indicator():
    np.testing.assert_array_equal(O.correctness([3, 1, 4, 1], [3, 1, 5, 9]), [1, 1, 0, 0])


# ------------------------------------------------------------------ the other two confidence metrics
def test_metrics_closed_forms():
    V = 37
    pm, mg = O.confidence_metrics(np.full((1, V), 2.5))
    assert abs(pm[0] - 1.0 / V) < 1e-15 and mg[0] == 0.0                  # uniform
    # one logit a above the rest: p1 = e^a / (e^a + V - 1), p2 = 1 / (e^a + V - 1)
    for a in (0.3, 2.0, 9.0):
        z = np.zeros(V)
        z[11] = a
        pm, mg = O.confidence_metrics(z)
        den = math.exp(a) + V - 1
        assert abs(pm[0] - math.exp(a) / den) < 1e-14 and abs(mg[0] - (math.exp(a) - 1) / den) < 1e-14
    # two-class case is the logistic function: p1 = sigma(|d|), margin = tanh(|d| / 2)
    for dlt in (0.0, 0.7, -3.0):
        pm, mg = O.confidence_metrics([0.0, dlt])
        assert abs(pm[0] - 1.0 / (1.0 + math.exp(-abs(dlt)))) < 1e-15
        assert abs(mg[0] - math.tanh(abs(dlt) / 2.0)) < 1e-15
    pm, mg = O.confidence_metrics([[4.2]])                                # a single class
    assert pm[0] == 1.0 and mg[0] == 1.0
    pm, mg = O.confidence_metrics([3.0, 3.0, 1.0])                        # tie at the top
    assert mg[0] == 0.0 and abs(pm[0] - 1.0 / (2.0 + math.exp(-2.0))) < 1e-15


def test_metrics_invariances_and_bounds():
    rng = np.random.default_rng(21)
    z = rng.normal(size=(30, 50)) * rng.uniform(0.1, 6.0, size=(30, 1))
    pm, mg = O.confidence_metrics(z)
    pm2, mg2 = O.confidence_metrics(z + 123.456)                           # shift
    np.testing.assert_allclose(pm2, pm, rtol=1e-12)
    np.testing.assert_allclose(mg2, mg, rtol=1e-10, atol=1e-14)
    perm = rng.permutation(50)
    pm3, mg3 = O.confidence_metrics(z[:, perm])                            # permutation
    np.testing.assert_allclose(pm3, pm, rtol=1e-13)
    np.testing.assert_allclose(mg3, mg, rtol=1e-11, atol=1e-15)
    assert ((pm >= 1.0 / 50 - 1e-15) & (pm <= 1.0)).all() and ((mg >= 0) & (mg <= pm)).all()
    H, lse, am, gap = O.softmax_stats(z)
    np.testing.assert_allclose(pm, np.exp(z[np.arange(30), am] - lse), rtol=1e-13)   # p of the argmax
    np.testing.assert_allclose(mg, pm * (1.0 - np.exp(-gap)), rtol=1e-11)            # from the logit gap
    assert (pm >= np.exp(-H) - 1e-12).all()                                # max p >= e^{-H}


def test_metrics_against_scipy_and_pure_python():
    from scipy.special import softmax
    rng = np.random.default_rng(4)
    z = rng.normal(size=(12, 9)) * 3.0
    pm, mg = O.confidence_metrics(z)
    p = softmax(z, axis=1)
    top = np.sort(p, axis=1)
    np.testing.assert_allclose(pm, top[:, -1], rtol=1e-13)
    np.testing.assert_allclose(mg, top[:, -1] - top[:, -2], rtol=1e-11, atol=1e-15)
    for r in range(3):                                                     # the formulas spelled out
        e = [math.exp(v) for v in z[r]]
        tot = sum(e)
        pr = sorted(v / tot for v in e)
        assert abs(pm[r] - pr[-1]) < 1e-14 and abs(mg[r] - (pr[-1] - pr[-2])) < 1e-14


def test_metrics_nan_row():
    pm, mg = O.confidence_metrics([[1.0, float("nan"), 0.0], [0.0, 1.0, 2.0]])
    assert np.isnan(pm[0]) and np.isnan(mg[0]) and np.isfinite(pm[1])


# ------------------------------------------------------------------ DSSD drafting
def test_dssd_draft_against_closed_form_exhaustively():
    """Every pattern of (exit layer, token) over 4 positions, 3 heads, tokens {0, 1=EOS}: the
    draft is the prefix of length min(limit, first fallback position, first drafted EOS + 1)."""
    n_heads, tau = 3, [1.0, 1.0, float("inf")]
    for limit in (1, 2, 3, 5):
        for exits in itertools.product(range(n_heads), repeat=4):
            for toks in itertools.product((0, 1), repeat=4):
                # entropies that make head `exits[t]` the first confident one (2 = none confident)
                H = [[0.5 if l >= e else 2.0 for l in range(n_heads)] for e in exits]
                T = [[7 if l != min(e, n_heads - 1) else tk for l in range(n_heads)] for e, tk in zip(exits, toks)]
                got = O.dssd_draft(H, T, tau, limit, eos_token=1)
                i_fb = next((t for t, e in enumerate(exits) if e == n_heads - 1), 99)
                i_eos = next((t for t, (e, tk) in enumerate(zip(exits, toks)) if t < i_fb and tk == 1), 99)
                L = min(limit, i_fb, i_eos + 1, 4)
                assert got["draft"] == list(toks[:L]) and got["exit_layer"] == list(exits[:L])
                want = ("eos" if L == i_eos + 1 else "limit" if L == limit else
                        "fallback" if L == i_fb else "exhausted")
                assert got["reason"] == want, (limit, exits, toks, got)
                assert got["fallback_token"] == (toks[i_fb] if want == "fallback" else -1)
                evals = sum(e + 1 for e in exits[:L]) + (n_heads if want == "fallback" else 0)
                assert got["n_evals"] == evals


def test_dssd_draft_special_cases():
    tau = [1.0, float("inf")]
    assert O.dssd_draft([[0.1, 0.1]], [[5, 6]], tau, 0, 9)["draft"] == []                 # no room
    r = O.dssd_draft([[float("nan"), 0.1]], [[5, 6]], tau, 4, 9)                           # NaN is not confident
    assert r["reason"] == "fallback" and r["fallback_token"] == 6 and r["draft"] == []
    r = O.dssd_draft([[1.0, 0.0]], [[5, 6]], tau, 4, 9)                                    # strict inequality
    assert r["reason"] == "fallback"
    r = O.dssd_draft([[0.2, 0.0]] * 3, [[5, 6]] * 3, tau, 8, 9)                            # positions run out
    assert r["draft"] == [5, 5, 5] and r["reason"] == "exhausted"


def test_dssd_draft_consistent_with_exit_rule_and_cascade():
    """Position by position the drafted (layer, token) is what exit_rule / cascade give."""
    rng = np.random.default_rng(12)
    d, V, n_heads, T = 16, 40, 4, 10
    Ws = [rng.normal(size=(V, d)) / math.sqrt(d) for _ in range(n_heads)]
    g = [np.ones(d)] * n_heads
    b = [np.zeros(d)] * n_heads
    h = rng.normal(size=(T, n_heads, d)) * rng.uniform(0.5, 6.0, size=(T, 1, 1))
    stats = [[O.head_eval(h[t, l][None, :], g[l], b[l], Ws[l]) for l in range(n_heads)] for t in range(T)]
    H = [[float(stats[t][l][0][0]) for l in range(n_heads)] for t in range(T)]
    tok = [[int(stats[t][l][2][0]) for l in range(n_heads)] for t in range(T)]
    tau = [float(np.median([H[t][l] for t in range(T)])) for l in range(n_heads - 1)] + [float("inf")]
    r = O.dssd_draft(H, tok, tau, limit=T, eos_token=-5)
    for t, (lay, tk) in enumerate(zip(r["exit_layer"], r["draft"])):
        assert lay == O.exit_rule(H[t], tau) and lay < n_heads - 1
        c = O.cascade([h[t, l][None, :] for l in range(n_heads)], g, b, Ws, tau)
        assert int(c["exit_layer"][0]) == lay and int(c["token"][0]) == tk
    if r["reason"] == "fallback":
        assert O.exit_rule(H[len(r["draft"])], tau) == n_heads - 1


# ---------------------------------------------------------------- verification bookkeeping
def _figures():
    rows = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "acceptance_figures.txt")):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            rows[f[0]] = [float(x) for x in f[1:]]
    return rows


def test_tally_reproduces_the_papers_printed_figures():
    """Section 4.3.2 prints rate and waste of two systems; with rate = accepted / drafted and
    wasted = drafted - accepted there must be integer token counts that print as those figures,
    and the printed ratios must follow from them."""
    fig = _figures()
    rates = {}
    for name in ("layerskip_best", "dssd_eps_0.9"):
        pct, wasted = fig[name]
        wasted = int(wasted)
        found = []
        for drafted in range(wasted, 100 * wasted):
            t = O.dssd_tally([drafted], [drafted - wasted])
            assert t["wasted"] == wasted and t["drafted"] == drafted and t["rounds"] == 1
            if abs(100.0 * t["acceptance_rate"] - pct) <= 0.05 + 1e-9:
                found.append((drafted, t["acceptance_rate"]))
        assert found, name                                  # the printed pair is attainable ...
        assert len(found) <= 2, (name, found)               # ... and pins the counts
        rates[name] = found[0][1]
        # the same counts under a wrong definition (waste over drafted, accepted over wasted+drafted)
        d = found[0][0]
        assert abs(100.0 * wasted / d - pct) > 1.0
        assert abs(100.0 * (d - wasted) / (d + wasted) - pct) > 1.0
    assert round(rates["dssd_eps_0.9"] / rates["layerskip_best"], 2) == fig["ratio_acceptance"][0]
    assert int(fig["layerskip_best"][1] / fig["dssd_eps_0.9"][1]) == int(fig["ratio_waste"][0])


def test_tally_against_token_by_token_enumeration():
    """Every drafted token is individually either committed (it and all before it match the
    model's prediction) or wasted; counting them one by one must give the tally of the
    verification's outputs."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        B, k = int(rng.integers(1, 6)), int(rng.integers(1, 7))
        draft = rng.integers(0, 2, size=(B, k))
        target = rng.integers(0, 2, size=(B, k + 1))
        lens = rng.integers(0, k + 1, size=B)
        layers = rng.integers(0, 24, size=(B, k))
        committed = wasted = lsum = 0
        for b in range(B):
            ok = True
            for j in range(int(lens[b])):
                ok = ok and draft[b, j] == target[b, j]
                committed += ok
                wasted += not ok
                lsum += int(layers[b, j])
        acc = [O.accepted_prefix(draft[b], target[b], int(lens[b])) for b in range(B)]
        t = O.dssd_tally(lens, acc, layers)
        assert (t["accepted"], t["wasted"], t["drafted"], t["rounds"], t["exit_layer_sum"]) == \
               (committed, wasted, int(lens.sum()), B, lsum)
        assert t["accepted"] + t["wasted"] == t["drafted"]
        if t["drafted"]:
            assert t["acceptance_rate"] == committed / t["drafted"]
        assert t["mean_accepted"] == committed / B


def test_tally_is_additive_and_handles_nothing_drafted():
    a = O.dssd_tally([3, 0, 5], [1, 0, 5], [[1, 2, 3, 9, 9], [9] * 5, [4] * 5])
    b = O.dssd_tally([2], [0], [[7, 8, 9, 9, 9]])
    ab = O.dssd_tally([3, 0, 5, 2], [1, 0, 5, 0], [[1, 2, 3, 9, 9], [9] * 5, [4] * 5, [7, 8, 9, 9, 9]])
    for key in ("rounds", "drafted", "accepted", "wasted", "exit_layer_sum"):
        assert a[key] + b[key] == ab[key]
    assert a["exit_layer_sum"] == 6 + 20 and b["exit_layer_sum"] == 15
    z = O.dssd_tally([0, 0], [0, 0])
    assert z["drafted"] == 0 and math.isnan(z["acceptance_rate"]) and z["mean_accepted"] == 0.0
    e = O.dssd_tally([], [])
    assert e["rounds"] == 0 and math.isnan(e["mean_accepted"])


# ---------------------------------------------------------------- training objectives (Section 3.3)
def test_kl_direction_and_two_class_values():
    """Hand-computed two-class values; the two directions differ, so a swapped operand fails."""
    zp, zq = np.log([0.5, 0.5]), np.log([0.9, 0.1])
    kl_pq, _ = O.token_losses(zp, zq)
    kl_qp, _ = O.token_losses(zq, zp)
    assert abs(kl_pq[0] - (0.5 * math.log(0.5 / 0.9) + 0.5 * math.log(0.5 / 0.1))) < 1e-14
    assert abs(kl_qp[0] - (0.9 * math.log(0.9 / 0.5) + 0.1 * math.log(0.1 / 0.5))) < 1e-14
    assert abs(kl_pq[0] - 0.5108256237659907) < 1e-12 and abs(kl_qp[0] - 0.3680642071684971) < 1e-12
    # logits, not probabilities, go in: a shift of either row of logits changes nothing
    kl_s, _ = O.token_losses(zp + 3.25, zq - 7.5)
    assert abs(kl_s[0] - kl_pq[0]) < 1e-13


def test_kl_against_scipy_and_gibbs():
    from scipy.special import rel_entr, softmax
    from scipy.stats import entropy
    rng = np.random.default_rng(3)
    zs = rng.normal(size=(40, 300)) * rng.uniform(0.1, 8.0, size=(40, 1))
    zt = rng.normal(size=(40, 300)) * rng.uniform(0.1, 8.0, size=(40, 1))
    kl, ce = O.token_losses(zs, zt)
    p, q = softmax(zs, axis=1), softmax(zt, axis=1)
    ref = rel_entr(p, q).sum(axis=1)                 # sum p log(p/q): the head's distribution first
    assert np.allclose(kl, ref, rtol=1e-10, atol=1e-12)
    assert np.allclose(kl, [entropy(p[t], q[t]) for t in range(40)], rtol=1e-10, atol=1e-12)
    assert not np.allclose(kl, rel_entr(q, p).sum(axis=1), rtol=1e-3)      # not the other direction
    assert (kl >= 0).all() and np.isnan(ce).all()
    same, _ = O.token_losses(zs, zs + 1.5)           # the same distribution: exactly no divergence
    assert np.abs(same).max() < 1e-13


def test_kl_from_uniform_is_logV_minus_entropy_golden():
    """Against the uniform distribution KL(y_hat || u) = ln V - H(y_hat): ties the loss to the
    closed-form entropies of the golden table."""
    for V, n, a, H_ref, _ in _golden_rows():
        z = np.zeros(V)
        z[:n] = a
        kl, _ = O.token_losses(z, np.full(V, -2.0))
        assert abs(kl[0] - (math.log(V) - H_ref)) < 1e-9 * max(1.0, math.log(V)), (V, n, a)


def test_kl_vanishing_probability_and_nonfinite():
    z = np.array([0.0, -2000.0, 1.0])                # exp underflows to exactly 0 for class 1
    kl, ce = O.token_losses(z, np.array([0.0, 5.0, 1.0]), labels=[2])
    p = np.exp([0.0, 1.0]) / (1.0 + math.e)
    lq = np.array([0.0, 1.0]) - math.log(1.0 + math.e ** 5 + math.e)
    assert abs(kl[0] - (p * (np.log(p) - lq)).sum()) < 1e-12
    assert abs(ce[0] + math.log(p[1])) < 1e-12
    kl, _ = O.token_losses(np.array([0.0, float("nan")]), np.array([0.0, 1.0]))
    assert np.isnan(kl[0])


def test_cross_entropy_values_and_relation_to_kl():
    rng = np.random.default_rng(8)
    V = 50
    zs = rng.normal(size=(30, V)) * 3
    labels = rng.integers(0, V, size=30)
    _, ce = O.token_losses(zs, zs, labels)
    lse = np.log(np.exp(zs).sum(axis=1))
    assert np.allclose(ce, lse - zs[np.arange(30), labels], rtol=1e-12)
    _, ce_u = O.token_losses(np.zeros((1, V)), np.zeros((1, V)), [7])
    assert abs(ce_u[0] - math.log(V)) < 1e-14         # uniform prediction: ln V whatever the label
    # CE against a label is the divergence of the label's (nearly) one-hot distribution from the
    # prediction, read in the other direction: KL(onehot || y_hat) = -log y_hat_label
    for t in range(5):
        onehot = np.full(V, -800.0)
        onehot[labels[t]] = 0.0
        kl_rev, _ = O.token_losses(onehot, zs[t])
        assert abs(kl_rev[0] - ce[t]) < 1e-10


def test_head_losses_means_and_hybrid():
    rng = np.random.default_rng(21)
    L, d, V = 12, 24, 70
    Ws, Wt = rng.normal(size=(V, d)) / 3, rng.normal(size=(V, d)) / 3
    g1, b1, g2, b2 = rng.normal(size=d), rng.normal(size=d), rng.normal(size=d), rng.normal(size=d)
    hs, ht = rng.normal(size=(L, d)) * 2, rng.normal(size=(L, d)) * 2
    labels = rng.integers(0, V, size=L)
    r = O.head_losses(hs, ht, g1, b1, Ws, g2, b2, Wt, labels, alpha=0.3)
    # per token it is the head evaluation's own logits: lse and entropy tie the two code paths
    zs = O.head_logits(O.layernorm(hs, g1, b1), Ws)
    zt = O.head_logits(O.layernorm(ht, g2, b2), Wt)
    H, lse, _, _ = O.softmax_stats(zs)
    _, lse_t, _, _ = O.softmax_stats(zt)
    ps = np.exp(zs - lse[:, None])
    cross = -(ps * (zt - lse_t[:, None])).sum(axis=1)            # cross-entropy H(y_hat, f)
    assert np.allclose(r["kl"], cross - H, rtol=1e-10, atol=1e-12)   # KL = H(p, q) - H(p)
    assert np.allclose(r["ce"], lse - zs[np.arange(L), labels], rtol=1e-12)
    assert abs(r["L_kl"] - r["kl"].mean()) < 1e-14 and abs(r["L_ce"] - r["ce"].mean()) < 1e-14
    assert abs(r["L_hyb"] - (0.3 * r["L_ce"] + 0.7 * r["L_kl"])) < 1e-14
    # the mean is over the sequence: repeating the sequence leaves every objective unchanged,
    # and the same head on the same hidden states as the model has no divergence from it
    r2 = O.head_losses(np.tile(hs, (2, 1)), np.tile(ht, (2, 1)), g1, b1, Ws, g2, b2, Wt, np.tile(labels, 2), 0.3)
    assert abs(r2["L_kl"] - r["L_kl"]) < 1e-13 and abs(r2["L_hyb"] - r["L_hyb"]) < 1e-13
    r0 = O.head_losses(hs, hs, g1, b1, Ws, g1, b1, Ws, labels, 1.0)
    assert abs(r0["L_kl"]) < 1e-13 and abs(r0["L_hyb"] - r0["L_ce"]) < 1e-14
    # bf16 mode rounds both heads' normalised activations, nothing else
    rb = O.head_losses(hs, ht, g1, b1, Ws, g2, b2, Wt, labels, 0.3, bf16=True)
    zs_b = O.head_logits(O.round_to_bf16(O.layernorm(hs, g1, b1)), Ws)
    zt_b = O.head_logits(O.round_to_bf16(O.layernorm(ht, g2, b2)), Wt)
    klb, ceb = O.token_losses(zs_b, zt_b, labels)
    assert np.array_equal(rb["kl"], klb) and np.array_equal(rb["ce"], ceb)
