"""Edge cases of the method on every kernel path, through the C ABI, against the oracle:
exact ties at the top (lowest index wins, eq. (2) with the build's tie rule), entropies exactly
on a threshold and beside it (strict H < tau, Sections 3.4.2 and 4.3.1), heads that start with
no live row, rows with NaN / Inf hidden states, the persistent kernel's give-up path, and the
calibration level met exactly (Section 3.4.1).

Row counts pick the kernel: at most 16 rows run the persistent kernel, more the batched ones
(bf16: 32-row blocks, one or two per wave; fp32: 16-row blocks); heads with a bias vector take
the plain streaming kernel at any row count.
"""
import math

import numpy as np
import pytest
import torch

from oracle import eh_oracle as O
from workloads import generators as G
from tests import parity_util as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
V_BIG = G.V_PYTHIA

# (lower, higher) vocabulary rows that are made to tie at the top, one pair per head.  With 256
# workgroups over 50304 rows a slice is 196.5 rows: the pairs sit in one 16-row tile, in one
# slice but different tiles, on both sides of the first slice boundary inside a tile (row 196
# cuts tile 12), in neighbouring slices and at the two ends of the vocabulary.
PAIRS_BIG = [(1000, 1003), (1010, 1100), (194, 198), (150, 250), (5, 50000), (50287, 50303)]


@pytest.fixture(scope="module")
def B():
    from paper_2407_21082_amd import binding
    return binding


def _outs(n):
    return (torch.full((n,), float("nan"), device=DEV), torch.full((n,), float("nan"), device=DEV),
            torch.full((n,), -7, dtype=torch.int32, device=DEV))


def _plant_ties(w, heads, hid, pairs, bf16, value=256.0):
    """Head l gets two identical vocabulary rows pairs[l] whose only non-zero weight is `value`
    at a hidden index where the LayerNorm output of most rows is clearly positive: their logit
    value * y_j is a single exact product on either side (no rounding, whatever the order of
    summation), equal for the two rows, and for those rows the largest by far."""
    wins = []
    for l, (a, b) in enumerate(pairs):
        y = O.layernorm(P.f64(hid.h[l]), P.f64(heads.gamma[l]), P.f64(heads.beta[l]), w.ln_eps, bf16_out=bf16)
        ok = y > 0.2
        j0 = int(np.argmax(ok.sum(axis=0) + 1000 * ok[0]))          # row 0 must be among them
        assert ok[0, j0] and ok[:, j0].sum() >= max(1, y.shape[0] // 4)
        heads.W[l][a].zero_()
        heads.W[l][a, j0] = value
        heads.W[l][b] = heads.W[l][a]
        wins.append(np.flatnonzero(ok[:, j0]))
    return wins


def _check_tie_head(name, got, orc, rows_tied, pair):
    """Statistics within tolerance everywhere, and on the rows where the oracle sees an exact
    tie of the planted pair at the top the index is the lower one -- no near-tie excuse."""
    H, lse, am = got
    H_o, lse_o, am_o, gap_o = orc
    P.compare_head(name, H, lse, am, orc, [])
    am = am.cpu().numpy()
    tied = [r for r in rows_tied if gap_o[r] == 0.0 and am_o[r] == pair[0]]
    assert len(tied) >= 1, f"{name}: the planted pair wins nowhere"
    for r in tied:
        assert am[r] == pair[0], f"{name}: row {r} picked {am[r]}, the tie {pair} goes to the lower index"
    return len(tied)


# ------------------------------------------------------------------ ties: eh_eval on every path
@pytest.mark.parametrize("dtype,d,rows", [("bf16", 1024, 16), ("bf16", 1024, 1), ("bf16", 256, 40), ("bf16", 256, 150),
                                          ("f32", 512, 16), ("f32", 512, 32)])
def test_exact_tie_at_the_top_goes_to_the_lower_index(B, dtype, d, rows):
    bf16 = dtype == "bf16"
    w = G.Workload("tie", d=d, V=V_BIG, n_heads=len(PAIRS_BIG), rows=rows, dtype=dtype, seed=700 + d + rows)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    wins = _plant_ties(w, heads, hid, PAIRS_BIG, bf16)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=rows)
    total = 0
    for l, pair in enumerate(PAIRS_BIG):
        H, lse, am = _outs(rows)
        B.eh_eval(ctx, l, hid.h[l], rows, H, lse, am)
        torch.cuda.synchronize()
        orc = P.oracle_head(hid.h[l], heads.gamma[l], heads.beta[l], heads.W[l], bf16)
        total += _check_tie_head(f"tie/{dtype}/{rows}/head{l}", (H, lse, am), orc, wins[l], pair)
    B.eh_check(ctx)
    B.eh_destroy(ctx)
    assert total >= len(PAIRS_BIG)


@pytest.mark.parametrize("rows", [9, 40])
def test_exact_tie_with_a_bias_vector(B, rows):
    pairs = [(100, 103), (7, 5100), (2047, 2049)]
    w = G.Workload("tiebias", d=128, V=5200, n_heads=len(pairs), rows=rows, dtype="bf16", seed=31 + rows)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    wins = _plant_ties(w, heads, hid, pairs, True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(9)
    bias = [torch.randn(w.V, generator=gen, device=DEV) for _ in pairs]
    for l, (a, b) in enumerate(pairs):
        bias[l][b] = bias[l][a]
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=rows, bias=bias)
    for l, pair in enumerate(pairs):
        H, lse, am = _outs(rows)
        B.eh_eval(ctx, l, hid.h[l], rows, H, lse, am)
        torch.cuda.synchronize()
        orc = O.head_eval(P.f64(hid.h[l]), P.f64(heads.gamma[l]), P.f64(heads.beta[l]), P.f64(heads.W[l]), 1e-5, True,
                          bias=P.f64(bias[l]))
        _check_tie_head(f"tiebias/{rows}/head{l}", (H, lse, am), orc, wins[l], pair)
    B.eh_destroy(ctx)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("Bsz,k", [(3, 3), (5, 4), (16, 8)])
def test_exact_tie_in_the_verification_targets(B, dtype, Bsz, k):
    """dssd_verify with ties at the top of the model's head: 12 positions (persistent-free small
    path), 25 and 144 (batched argmax-only kernel, one and two blocks per wave)."""
    bf16 = dtype == "bf16"
    rows = Bsz * (k + 1)
    pair = (1200, 30000)
    w = G.Workload("tiever", d=256, V=V_BIG, n_heads=1, rows=rows, dtype=dtype, seed=11 * Bsz + k)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV, amp=torch.full((rows,), 1.5))    # every other row decides clearly
    _plant_ties(w, heads, hid, [pair], bf16)
    f_final = hid.h[0].reshape(Bsz, k + 1, w.d).contiguous()
    f64 = P.f64
    _, _, tgt_o, gap_o = O.dssd_verify(f64(f_final), np.zeros((Bsz, k), dtype=np.int64), f64(heads.gamma[0]),
                                       f64(heads.beta[0]), f64(heads.W[0]), None, 1e-5, bf16)
    # drafts: the model's own targets with every fifth one changed, so prefixes of all lengths occur
    draft = tgt_o[:, :k].copy()
    flat = draft.reshape(-1)
    flat[2::5] = (flat[2::5] + 1) % w.V
    acc_o, nxt_o, tgt_o, gap_o = O.dssd_verify(f64(f_final), draft, f64(heads.gamma[0]), f64(heads.beta[0]),
                                               f64(heads.W[0]), None, 1e-5, bf16)
    tied = np.flatnonzero((gap_o.reshape(-1) == 0.0) & (tgt_o.reshape(-1) == pair[0]))
    assert len(tied) >= 1
    assert (np.delete(gap_o.reshape(-1), tied) > 1e-3).all()
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")], max_rows=rows)
    acc = torch.full((Bsz,), -1, dtype=torch.int32, device=DEV)
    nxt = torch.full((Bsz,), -1, dtype=torch.int32, device=DEV)
    tgt = torch.full((Bsz, k + 1), -1, dtype=torch.int32, device=DEV)
    B.dssd_verify(ctx, f_final, torch.from_numpy(draft).to(torch.int32).to(DEV).contiguous(), None, acc, nxt, tgt)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tgt.cpu().numpy(), tgt_o)
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), nxt_o)
    B.eh_destroy(ctx)


# ------------------------------------------------------------------ the exit test at the threshold
def _f32(x):
    return float(np.float32(x))


def test_exit_decide_on_exact_boundary_entropies(B):
    """eh_exit_decide takes the entropies from the caller, so values on the threshold, one unit in
    the last place beside it, NaN, the infinities and the two zeros can be fed exactly; the rule is
    the oracle's exit_rule (strict H < tau; the last head always answers)."""
    taus = [1.5, 0.0, float("-inf"), float("inf"), 0.25]
    w = G.Workload("decide", d=64, V=64, n_heads=len(taus), rows=4, dtype="bf16", seed=3)
    heads = G.make_heads(w, DEV)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, taus, max_rows=400)
    up = lambda x: _f32(np.nextafter(np.float32(x), np.float32(np.inf)))
    dn = lambda x: _f32(np.nextafter(np.float32(x), np.float32(-np.inf)))
    vals = [1.5, up(1.5), dn(1.5), 0.0, -0.0, up(0.0), dn(0.0), float("nan"), float("inf"), float("-inf"),
            0.25, up(0.25), dn(0.25), 3.0e38, -3.0e38, 1e-45, -1e-45, 0.7, 2.0, -1.0]
    rng = np.random.default_rng(5)
    Hh = np.array(vals * 15, dtype=np.float32)             # 300 positions: more than one sweep of the workgroup
    rng.shuffle(Hh)
    n = len(Hh)
    H = torch.from_numpy(Hh).to(DEV)
    am = torch.arange(1000, 1000 + n, dtype=torch.int32, device=DEV)
    perm = torch.from_numpy(rng.permutation(n).astype(np.int32)).to(DEV)
    for head in range(len(taus)):
        for idx, n_dev in ((None, None), (perm, None), (perm, 173), (None, 0)):
            ex = torch.full((n,), -1, dtype=torch.int32, device=DEV)
            tok = torch.full((n,), -1, dtype=torch.int32, device=DEV)
            act = torch.full((n,), -9, dtype=torch.int32, device=DEV)
            cnt = torch.full((1,), -9, dtype=torch.int32, device=DEV)
            nd = None if n_dev is None else torch.tensor([n_dev], dtype=torch.int32, device=DEV)
            B.eh_exit_decide(ctx, head, H, am, n, ex, tok, act, cnt, row_idx=idx, n_rows_dev=nd)
            torch.cuda.synchronize()
            live = n if n_dev is None else n_dev
            want_ex = np.full(n, -1)
            want_tok = np.full(n, -1)
            stay = []
            for p in range(live):
                r = p if idx is None else int(perm[p])
                # the oracle's rule on a two-head stack: this head, then one that always answers
                leaves = head == len(taus) - 1 or O.exit_rule([float(Hh[p]), 0.0], [taus[head], math.inf]) == 0
                if leaves:
                    want_ex[r], want_tok[r] = head, 1000 + p
                else:
                    stay.append(r)
            np.testing.assert_array_equal(ex.cpu().numpy(), want_ex)
            np.testing.assert_array_equal(tok.cpu().numpy(), want_tok)
            assert int(cnt.item()) == len(stay) and act[:len(stay)].tolist() == stay, (head, n_dev)
    B.eh_destroy(ctx)


@pytest.mark.parametrize("dtype,rows", [("bf16", 8), ("bf16", 40), ("bf16", 150), ("f32", 12), ("f32", 40)])
def test_cascade_is_strict_at_its_own_entropy(B, dtype, rows):
    """The exit test inside the cascade kernels (persistent kernel; cascade step kernel behind the
    batched ones): the threshold of head 0 is set to the very float the library reports as a row's
    entropy, and to its two neighbours.  Equal or below: the row goes on; one unit above: it leaves."""
    w = G.Workload("strict", d=256, V=3000, n_heads=3, rows=rows, dtype=dtype, seed=rows + 40)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    # the library's own entropies of every head on every row: a cascade in which no exit head ever
    # fires reports them all (the same kernels, hence the same floats, as the cascades below)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("-inf"), float("-inf"), 0.0], max_rows=rows)
    Hg = torch.zeros((3, rows), device=DEV)
    Ag = torch.zeros((3, rows), dtype=torch.int32, device=DEV)
    ex0 = torch.full((rows,), -1, dtype=torch.int32, device=DEV)
    tok0 = torch.full((rows,), -1, dtype=torch.int32, device=DEV)
    B.eh_cascade(ctx, hid.h, rows, ex0, tok0, Hg, None)
    for l in range(3):
        B.eh_eval(ctx, l, hid.h[l], rows, None, None, Ag[l])
    torch.cuda.synchronize()
    assert (ex0 == 2).all() and torch.equal(tok0, Ag[2]) and torch.isfinite(Hg).all()
    B.eh_destroy(ctx)
    Hn, An = Hg.cpu().numpy(), Ag.cpu().numpy()
    r_star = int(np.argsort(Hn[0])[rows // 2])              # a row in the middle of head 0's entropies
    h0 = np.float32(Hn[0, r_star])
    for tau0, leaves in ((h0, False), (np.nextafter(h0, np.float32(-np.inf)), False),
                         (np.nextafter(h0, np.float32(np.inf)), True)):
        tau = [float(tau0), float("-inf"), float("inf")]
        ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=rows)
        ex = torch.full((rows,), -1, dtype=torch.int32, device=DEV)
        tok = torch.full((rows,), -1, dtype=torch.int32, device=DEV)
        Hout = torch.zeros((3, rows), device=DEV)
        nev = torch.zeros(1, dtype=torch.int64, device=DEV)
        B.eh_cascade(ctx, hid.h, rows, ex, tok, Hout, nev)
        torch.cuda.synchronize()
        B.eh_check(ctx)
        B.eh_destroy(ctx)
        want = np.array([O.exit_rule([float(Hn[l, r]) for l in range(3)], tau) for r in range(rows)])
        np.testing.assert_array_equal(ex.cpu().numpy(), want)
        assert (want[r_star] == 0) == leaves
        np.testing.assert_array_equal(tok.cpu().numpy(), An[want, np.arange(rows)])
        Ho = Hout.cpu().numpy()
        # head 0 sees the same columns in both cascades: the same floats.  Later heads see the
        # survivors compacted, and a different number of token blocks per wave may round the last bit
        # differently; beyond the exit nothing is evaluated.
        assert (Ho[0] == Hn[0]).all()
        for r in range(rows):
            assert np.allclose(Ho[1:want[r] + 1, r], Hn[1:want[r] + 1, r], rtol=2e-6, atol=2e-6)
            assert np.isnan(Ho[want[r] + 1:, r]).all()
        assert int(nev.item()) == int((want + 1).sum())


# ------------------------------------------------------------------ heads that start with no live row
@pytest.mark.parametrize("dtype,rows", [("bf16", 70), ("bf16", 150), ("bf16", 12), ("f32", 40)])
def test_cascade_with_heads_that_have_no_live_row(B, dtype, rows):
    bf16 = dtype == "bf16"
    w = G.Workload("empty", d=128, V=2000, n_heads=5, rows=rows, dtype=dtype, seed=rows + 5, kappa=0.6)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    full = P.oracle_all_heads(heads, hid.h, bf16)
    srt = np.sort(full[0][0])
    i = max(range(rows // 3, 2 * rows // 3), key=lambda j: srt[j] - srt[j - 1])    # the widest gap near the middle
    med = float(srt[i] + srt[i - 1]) / 2
    assert np.abs(full[0][0] - med).min() > 2e-3
    f64 = P.f64
    for name, tau in (("all leave at head 0", [float("inf")] * 5),
                      ("half at head 0, the rest at head 2", [med, float("-inf"), float("inf"), 1.0, float("inf")])):
        ref = O.cascade([f64(hid.h[l]) for l in range(5)], [f64(g) for g in heads.gamma], [f64(b) for b in heads.beta],
                        [f64(W) for W in heads.W], tau, 1e-5, bf16)
        assert ref["exit_layer"].max() <= 2
        ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=rows)
        for repeat in range(2):                               # the second call meets the first one's leftovers
            ex = torch.full((rows,), -1, dtype=torch.int32, device=DEV)
            tok = torch.full((rows,), -1, dtype=torch.int32, device=DEV)
            Hout = torch.full((5, rows), 7.0, device=DEV)
            nev = torch.zeros(1, dtype=torch.int64, device=DEV)
            B.eh_cascade(ctx, hid.h, rows, ex, tok, Hout, nev)
            torch.cuda.synchronize()
            B.eh_check(ctx)
            np.testing.assert_array_equal(ex.cpu().numpy(), ref["exit_layer"], err_msg=name)
            bad = np.flatnonzero(tok.cpu().numpy() != ref["token"])
            assert all(ref["gap"][ref["exit_layer"][r], r] < P.NEAR_TIE for r in bad), name
            Hg = Hout.double().cpu().numpy()
            seen = ~np.isnan(ref["H"])
            np.testing.assert_array_equal(~np.isnan(Hg), seen, err_msg=name)
            assert np.abs(Hg[seen] - ref["H"][seen]).max() <= P.TOL_H
            assert int(nev.item()) == int(seen.sum()) == int((ref["exit_layer"] + 1).sum())
        B.eh_destroy(ctx)


# ------------------------------------------------------------------ NaN / Inf hidden states
@pytest.mark.parametrize("dtype,rows", [("bf16", 40), ("bf16", 150), ("bf16", 9), ("f32", 40), ("f32", 9)])
def test_nan_and_inf_rows_have_defined_outputs(B, dtype, rows):
    """A hidden state with a NaN or an Inf in it: NaN entropy and log-sum-exp, argmax -1, never
    through the exit test; every other row is untouched.  The oracle says the same."""
    bf16 = dtype == "bf16"
    w = G.Workload("nan", d=128, V=3000, n_heads=3, rows=rows, dtype=dtype, seed=rows + 77, kappa=0.6)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    bad_nan, bad_inf, bad_last = 2, rows - 1, 5
    hid.h[0, bad_nan, 17] = float("nan")
    hid.h[0, bad_inf, 0] = float("inf")
    hid.h[1, bad_inf, 3] = float("-inf")
    hid.h[:, bad_last, 100] = float("nan")                    # NaN at every head: token -1 at the last
    tau = [1e9, 1e9, float("inf")]                              # every finite entropy exits at head 0
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=rows)
    for l in range(3):
        H, lse, am = _outs(rows)
        B.eh_eval(ctx, l, hid.h[l], rows, H, lse, am)
        torch.cuda.synchronize()
        orc = P.oracle_head(hid.h[l], heads.gamma[l], heads.beta[l], heads.W[l], bf16)
        nan_o = np.isnan(orc[0])
        assert nan_o.sum() == (3 if l == 0 else 2 if l == 1 else 1)
        np.testing.assert_array_equal(torch.isnan(H).cpu().numpy(), nan_o)
        np.testing.assert_array_equal(torch.isnan(lse).cpu().numpy(), nan_o)
        assert (am.cpu().numpy()[nan_o] == -1).all() and (orc[2][nan_o] == -1).all()
        keep = torch.from_numpy(np.flatnonzero(~nan_o)).to(DEV)
        P.compare_head(f"nan/{dtype}/{rows}/head{l}", H[keep], lse[keep], am[keep], tuple(x[~nan_o] for x in orc), [])
    f64 = P.f64
    ref = O.cascade([f64(hid.h[l]) for l in range(3)], [f64(g) for g in heads.gamma], [f64(b) for b in heads.beta],
                    [f64(W) for W in heads.W], tau, 1e-5, bf16)
    assert ref["exit_layer"][bad_nan] == 1 and ref["exit_layer"][bad_inf] == 2 and ref["token"][bad_last] == -1
    ex = torch.full((rows,), -1, dtype=torch.int32, device=DEV)
    tok = torch.full((rows,), -7, dtype=torch.int32, device=DEV)
    B.eh_cascade(ctx, hid.h, rows, ex, tok, None, None)
    torch.cuda.synchronize()
    B.eh_check(ctx)
    np.testing.assert_array_equal(ex.cpu().numpy(), ref["exit_layer"])
    badtok = np.flatnonzero(tok.cpu().numpy() != ref["token"])
    assert all(ref["gap"][ref["exit_layer"][r], r] < P.NEAR_TIE for r in badtok)
    assert int(tok[bad_last].item()) == -1
    B.eh_destroy(ctx)


@pytest.mark.parametrize("Bsz,k", [(2, 3), (6, 4)])
def test_verify_with_a_nan_position(B, Bsz, k):
    rows = Bsz * (k + 1)
    w = G.Workload("nanver", d=128, V=3000, n_heads=1, rows=rows, dtype="bf16", seed=rows)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV, amp=torch.full((rows,), 1.5))
    f_final = hid.h[0].reshape(Bsz, k + 1, w.d).contiguous()
    f_final[1, 2, 9] = float("nan")
    f64 = P.f64
    _, _, tgt0, _ = O.dssd_verify(f64(f_final), np.zeros((Bsz, k), dtype=np.int64), f64(heads.gamma[0]),
                                  f64(heads.beta[0]), f64(heads.W[0]), None, 1e-5, True)
    draft = tgt0[:, :k].copy()                                  # all drafts right: row 1 stops at the NaN position
    draft[1, 2] = 0
    acc_o, nxt_o, tgt_o, gap_o = O.dssd_verify(f64(f_final), draft, f64(heads.gamma[0]), f64(heads.beta[0]),
                                               f64(heads.W[0]), None, 1e-5, True)
    assert tgt_o[1, 2] == -1 and acc_o[1] == 2 and nxt_o[1] == -1 and acc_o[0] == k
    assert np.nanmin(gap_o) > 1e-3
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")], max_rows=rows)
    acc = torch.full((Bsz,), -5, dtype=torch.int32, device=DEV)
    nxt = torch.full((Bsz,), -5, dtype=torch.int32, device=DEV)
    tgt = torch.full((Bsz, k + 1), -5, dtype=torch.int32, device=DEV)
    B.dssd_verify(ctx, f_final, torch.from_numpy(draft).to(torch.int32).to(DEV).contiguous(), None, acc, nxt, tgt)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tgt.cpu().numpy(), tgt_o)
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), nxt_o)
    B.eh_destroy(ctx)


# ------------------------------------------------------------------ the persistent kernel gives up and recovers
def test_persistent_kernel_gives_up_cleanly_and_recovers(B):
    """With the bound of its waits set to zero polls a workgroup gives up at the first record of
    another workgroup that is not there yet: every kernel still ends, eh_check reports the failure
    once, rows that were not finished read -1 / NaN, and the next call on the context is normal."""
    w = G.scaled(G.CONFIGS["c1_decode"], n_heads=6, rows=8)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    tau = G.tau_linear(w)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=8)

    def cascade():
        ex = torch.full((8,), -7, dtype=torch.int32, device=DEV)
        tok = torch.full((8,), -7, dtype=torch.int32, device=DEV)
        Hout = torch.full((6, 8), 5.0, device=DEV)
        B.eh_cascade(ctx, hid.h, 8, ex, tok, Hout, None)
        torch.cuda.synchronize()
        return ex.cpu().numpy(), tok.cpu().numpy(), Hout.cpu().numpy()

    good = cascade()
    B.eh_check(ctx)
    assert (good[0] >= 0).all() and (good[1] >= 0).all()
    B.eh_set_spin_limit(ctx, 0)
    failures = 0
    for _ in range(3):
        ex, tok, Hout = cascade()
        try:
            B.eh_check(ctx)
        except B.EhError as e:
            failures += 1
            assert e.status == 5
        for r in range(8):                                    # finished rows are right, the others preset
            assert (ex[r], tok[r]) in ((-1, -1), (good[0][r], good[1][r]))
        same = (Hout == good[2]) | (np.isnan(Hout))
        assert same.all()
        B.eh_check(ctx)                                       # reported once, then cleared
    assert failures >= 1, "zero polls never made a workgroup give up"
    H, lse, am = _outs(8)
    B.eh_eval(ctx, 2, hid.h[2], 8, H, lse, am)                # evaluation mode presets NaN / -1
    torch.cuda.synchronize()
    try:
        B.eh_check(ctx)
        assert torch.isfinite(H).all() and (am >= 0).all()
    except B.EhError:
        assert ((am == -1) | (am >= 0)).all() and (torch.isnan(H) | torch.isfinite(H)).all()
    B.eh_set_spin_limit(ctx, 1 << 22)
    again = cascade()
    B.eh_check(ctx)
    assert all(np.array_equal(a, b, equal_nan=True) for a, b in zip(good, again))
    with pytest.raises(B.EhError):
        B.eh_set_spin_limit(ctx, -1)
    B.eh_destroy(ctx)


@pytest.mark.parametrize("mode", ["cascade", "verify"])
def test_rows_kernel_gives_up_cleanly_and_recovers(B, mode):
    """The same for the persistent kernel behind 17 .. 256 rows (cascade and verification)."""
    w = G.Workload("giveup", d=256, V=20000, n_heads=5, rows=48, dtype="bf16", seed=8, kappa=0.6)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=48)
    f_final = hid.h[4].reshape(6, 8, w.d).contiguous()
    gen = torch.Generator(device="cpu")
    gen.manual_seed(1)
    draft = torch.randint(0, w.V, (6, 7), generator=gen).to(torch.int32).to(DEV)

    def run():
        if mode == "cascade":
            a = torch.full((48,), -7, dtype=torch.int32, device=DEV)
            b = torch.full((48,), -7, dtype=torch.int32, device=DEV)
            B.eh_cascade(ctx, hid.h, 48, a, b, None, None)
        else:
            a = torch.full((6,), -7, dtype=torch.int32, device=DEV)
            b = torch.full((6,), -7, dtype=torch.int32, device=DEV)
            B.dssd_verify(ctx, f_final, draft, None, a, b, None)
        torch.cuda.synchronize()
        return a.cpu().numpy(), b.cpu().numpy()

    good = run()
    B.eh_check(ctx)
    assert (good[0] >= 0).all() and (good[1] >= 0).all()
    B.eh_set_spin_limit(ctx, 0)
    failures = 0
    for _ in range(3):
        a, b = run()
        try:
            B.eh_check(ctx)
        except B.EhError as e:
            failures += 1
            assert e.status == 5
        for i in range(len(a)):                               # finished rows are right, the others preset
            assert (a[i], b[i]) in ((-1, -1), (good[0][i], good[1][i]))
    assert failures >= 1, "zero polls never made a workgroup give up"
    B.eh_set_spin_limit(ctx, 1 << 22)
    again = run()
    B.eh_check(ctx)
    assert np.array_equal(good[0], again[0]) and np.array_equal(good[1], again[1])
    B.eh_destroy(ctx)


# ------------------------------------------------------------------ calibration level met exactly
def test_calibrate_level_at_the_boundary(B):
    w = G.Workload("calib", d=64, V=64, n_heads=1, rows=4, dtype="bf16", seed=1)
    heads = G.make_heads(w, DEV)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")], max_rows=4)
    for eps, n, c in ((0.7, 10, 7), (0.01, 100, 1), (0.55, 20, 11), (0.02, 50, 1), (0.07, 100, 7), (0.4, 5, 2),
                      (0.3, 10, 3), (0.1, 10, 1), (0.9, 10, 9), (0.6, 5, 3), (1.0, 9, 9)):
        levels = [eps, min(1.0, float(np.nextafter(eps, 2.0))), float(np.nextafter(eps, -1.0))]
        for correct in (c, c - 1):
            H = torch.full((n,), 1.25, device=DEV)
            ref = torch.zeros(n, dtype=torch.int32, device=DEV)
            pred = torch.tensor([0] * correct + [1] * (n - correct), dtype=torch.int32, device=DEV)
            tau = torch.zeros(3, device=DEV)
            cnt = torch.zeros(3, dtype=torch.int64, device=DEV)
            B.eh_calibrate(ctx, H, pred, ref, levels, tau, cnt)
            torch.cuda.synchronize()
            t = O.correctness(pred.cpu().numpy(), ref.cpu().numpy())
            for i, e in enumerate(levels):
                want = O.calibrate_threshold(H.double().cpu().numpy(), t, e)
                assert (float(tau[i]), int(cnt[i])) == want, (eps, n, correct, i)
    B.eh_destroy(ctx)


# ------------------------------------------------------------------ few rows, hidden size above 2048
@pytest.mark.parametrize("rows", [1, 9, 16])
def test_few_rows_of_a_wide_model_run_the_persistent_cascade(B, rows):
    """The single-launch kernel for at most 16 rows stops at hidden size 2048; beyond it (the 2.8B
    shape of the batched configurations has 2560) a cascade or a verification of few rows is served
    by the kernel for up to 256 rows, in one launch as well.  Parity as for any cascade; that it is
    that kernel which ran shows in its bounded wait giving up when told to poll zero times."""
    w = G.Workload("wide", d=2176, V=3000, n_heads=5, rows=rows, dtype="bf16", seed=40 + rows, kappa=0.6)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    n = w.n_heads
    full = P.oracle_all_heads(heads, hid.h, True)
    tau = G.tau_for_schedule(full[0], n) if rows > 1 else G.tau_linear(w)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=rows)
    ex = torch.full((rows,), -7, dtype=torch.int32, device=DEV)
    tok = torch.full((rows,), -7, dtype=torch.int32, device=DEV)
    Hout = torch.zeros((n, rows), device=DEV)
    nev = torch.zeros(1, dtype=torch.int64, device=DEV)
    B.eh_cascade(ctx, hid.h, rows, ex, tok, Hout, nev)
    torch.cuda.synchronize()
    B.eh_check(ctx)
    P.compare_cascade(f"wide{rows}", ex, tok, Hout, full[0], full[2], full[3], tau, [])
    assert int(nev.item()) == int((ex.long() + 1).sum().item())
    # verification of the same rows as one draft row of rows - 1 tokens (final head)
    k = rows - 1
    fin = n - 1
    f_final = hid.h[fin].reshape(1, rows, w.d).contiguous()
    target_o = full[2][fin]                                          # the oracle's argmax per position
    draft = torch.tensor(target_o[:k].reshape(1, k), dtype=torch.int32, device=DEV)
    if k >= 3:
        draft[0, k // 2] = (int(target_o[k // 2]) + 1) % w.V          # first mismatch in the middle
    acc = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    nxt = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    tgt = torch.full((rows,), -7, dtype=torch.int32, device=DEV)
    B.dssd_verify(ctx, f_final, draft, None, acc, nxt, tgt)
    torch.cuda.synchronize()
    B.eh_check(ctx)
    near = full[3][fin] < P.NEAR_TIE
    assert all(int(tgt[i]) == int(target_o[i]) or near[i] for i in range(rows))
    if not near.any():
        want = k // 2 if k >= 3 else k
        assert int(acc.item()) == want and int(nxt.item()) == int(target_o[want])
    # the persistent kernel, not the launch-per-head path: only it can give up
    B.eh_set_spin_limit(ctx, 0)
    gave_up = 0
    for _ in range(3):
        B.eh_cascade(ctx, hid.h, rows, ex, tok, None, None)
        try:
            B.eh_check(ctx)
        except B.EhError:
            gave_up += 1
    assert gave_up >= 1
    B.eh_set_spin_limit(ctx, 1 << 22)
    ex2 = torch.full((rows,), -7, dtype=torch.int32, device=DEV)
    tok2 = torch.full((rows,), -7, dtype=torch.int32, device=DEV)
    B.eh_cascade(ctx, hid.h, rows, ex2, tok2, None, None)
    torch.cuda.synchronize()
    B.eh_check(ctx)
    P.compare_cascade(f"wide{rows}b", ex2, tok2, None, full[0], full[2], full[3], tau, [])
    B.eh_destroy(ctx)


# ------------------------------------------------------------------ every block layout of the rows kernel
@pytest.mark.parametrize("rows", [17, 33, 97, 129, 161, 193, 225, 256])
def test_cascade_across_block_layouts(B, rows):
    """1 to 8 blocks of 32 rows on the four waves of the kernel for 17 .. 256 rows (no block, one
    or two per wave), shrinking from head to head as rows leave on the 10 / 40 / 70 % schedule, so
    that the layout changes inside one launch; the oracle on every row, and the same launch
    twice for a bitwise repeat (the list of live rows is built through atomics)."""
    w = G.Workload("blocks", d=160, V=2500, n_heads=7, rows=rows, dtype="bf16", seed=900 + rows, kappa=0.6)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    n = w.n_heads
    full = P.oracle_all_heads(heads, hid.h, True)
    tau = G.tau_for_schedule(full[0], n)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=rows)
    outs = []
    for _ in range(2):
        ex = torch.full((rows,), -7, dtype=torch.int32, device=DEV)
        tok = torch.full((rows,), -7, dtype=torch.int32, device=DEV)
        Hout = torch.zeros((n, rows), device=DEV)
        nev = torch.zeros(1, dtype=torch.int64, device=DEV)
        B.eh_cascade(ctx, hid.h, rows, ex, tok, Hout, nev)
        torch.cuda.synchronize()
        B.eh_check(ctx)
        outs.append((ex, tok, Hout, nev))
    ex, tok, Hout, nev = outs[0]
    P.compare_cascade(f"blocks{rows}", ex, tok, Hout, full[0], full[2], full[3], tau, [])
    assert int(nev.item()) == int((ex.long() + 1).sum().item())
    assert len(set(ex.tolist())) >= 4
    assert torch.equal(ex, outs[1][0]) and torch.equal(tok, outs[1][1])
    assert torch.equal(Hout.view(torch.int32), outs[1][2].view(torch.int32))
    B.eh_destroy(ctx)
