"""GPU-vs-oracle parity, through the C ABI, on seeded synthetic inputs.

Small ragged shapes exercise tile tails and every launch variant; the five
workload configurations then run at their real sizes, compared either in full
or on a stated sample of rows/steps the oracle can afford.
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
TOL_P = 2e-4   # a probability moves by at most p(1-p) <= 1/4 of a logit error; logits carry fp32


@pytest.fixture(scope="module")
def B():
    from paper_2407_21082_amd import binding
    return binding


def _outs(n):
    return (torch.full((n,), float("nan"), device=DEV), torch.full((n,), float("nan"), device=DEV),
            torch.full((n,), -7, dtype=torch.int32, device=DEV))


def _eval_all(B, ctx, heads, hid, R, bf16, name, log, rows=None):
    for l in range(len(heads.W)):
        H, lse, am = _outs(R)
        B.eh_eval(ctx, l, hid.h[l], R, H, lse, am)
        torch.cuda.synchronize()
        sel = slice(None) if rows is None else rows
        orc = P.oracle_head(hid.h[l][sel], heads.gamma[l], heads.beta[l], heads.W[l], bf16)
        P.compare_head(f"{name}/head{l}", H[sel], lse[sel], am[sel], orc, log)


# --------------------------------------------------------------- small shapes
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V,d,R", [(1000, 200, 1), (1000, 200, 5), (4099 - 3, 96, 17), (777, 512, 37),
                                    (2048, 256, 161), (16, 32, 16), (50, 8, 3), (1500, 160, 1000), (33, 64, 33)])
def test_small_ragged_shapes(B, dtype, V, d, R):
    if dtype == "f32" and d % 4:
        pytest.skip("d must hold whole 16-byte groups")
    w = G.Workload("small", d=d, V=V, n_heads=3, rows=R, dtype=dtype, seed=V * 31 + d + R)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=R)
    log = []
    _eval_all(B, ctx, heads, hid, R, dtype == "bf16", f"small{V}x{d}x{R}", log)
    B.eh_destroy(ctx)


def test_bias_and_strided_rows(B):
    w = G.Workload("bias", d=128, V=520, n_heads=1, rows=9, dtype="bf16", seed=5)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    gen = torch.Generator(device=DEV); gen.manual_seed(3)
    bias = [torch.randn(w.V, generator=gen, device=DEV) * 2]
    wide = torch.zeros((9, 256), dtype=torch.bfloat16, device=DEV)
    wide[:, :128] = hid.h[0]
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")], max_rows=16, bias=bias)
    H, lse, am = _outs(9)
    B.eh_eval(ctx, 0, wide, 9, H, lse, am, row_stride=256)
    torch.cuda.synchronize()
    orc = O.head_eval(P.f64(hid.h[0]), P.f64(heads.gamma[0]), P.f64(heads.beta[0]), P.f64(heads.W[0]),
                      1e-5, True, bias=P.f64(bias[0]))
    P.compare_head("bias", H, lse, am, orc, [])
    B.eh_destroy(ctx)


def test_gather_and_device_row_count(B):
    w = G.Workload("gather", d=256, V=3000, n_heads=1, rows=40, dtype="bf16", seed=11)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")], max_rows=40)
    idx = torch.tensor([39, 0, 7, 7, 21, 3, 38, 12, 1, 30, 2], dtype=torch.int32, device=DEV)
    n_dev = torch.tensor([9], dtype=torch.int32, device=DEV)        # only the first 9 are live
    H, lse, am = _outs(11)
    B.eh_eval(ctx, 0, hid.h[0], 11, H, lse, am, row_idx=idx, n_rows_dev=n_dev)
    torch.cuda.synchronize()
    sel = idx[:9].long()
    orc = P.oracle_head(hid.h[0][sel], heads.gamma[0], heads.beta[0], heads.W[0], True)
    P.compare_head("gather", H[:9], lse[:9], am[:9], orc, [])
    assert torch.isnan(H[9:]).all() and (am[9:] == -7).all()     # dead positions untouched
    # the same through the batched kernel (more than 16 positions): 40 positions, 25 live
    gen = torch.Generator(device="cpu")
    gen.manual_seed(5)
    idx = torch.randint(0, 40, (40,), generator=gen).to(torch.int32).to(DEV)
    n_dev = torch.tensor([25], dtype=torch.int32, device=DEV)
    H, lse, am = _outs(40)
    B.eh_eval(ctx, 0, hid.h[0], 40, H, lse, am, row_idx=idx, n_rows_dev=n_dev)
    torch.cuda.synchronize()
    sel = idx[:25].long()
    orc = P.oracle_head(hid.h[0][sel], heads.gamma[0], heads.beta[0], heads.W[0], True)
    P.compare_head("gather40", H[:25], lse[:25], am[:25], orc, [])
    assert torch.isnan(H[25:]).all() and (am[25:] == -7).all()
    B.eh_destroy(ctx)


def test_exit_decide_and_manual_cascade_equals_eh_cascade(B):
    w = G.Workload("casc", d=128, V=2000, n_heads=6, rows=70, dtype="bf16", seed=17, kappa=0.6)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    R, n = w.rows, w.n_heads
    full = P.oracle_all_heads(heads, hid.h, True)
    tau = G.tau_for_schedule(full[0], n)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=R)
    # library cascade
    ex = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    tok = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    Hout = torch.zeros((n, R), device=DEV)
    nev = torch.zeros(1, dtype=torch.int64, device=DEV)
    B.eh_cascade(ctx, hid.h, R, ex, tok, Hout, nev)
    torch.cuda.synchronize()
    log = []
    P.compare_cascade("casc", ex, tok, Hout, full[0], full[2], full[3], tau, log)
    assert len(set(ex.tolist())) >= 4
    assert int(nev.item()) == int((ex.long() + 1).sum().item())
    # the same thing through eh_eval + eh_exit_decide
    ex2 = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    tok2 = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    act = [torch.zeros(R, dtype=torch.int32, device=DEV) for _ in range(2)]
    cnt = [torch.zeros(1, dtype=torch.int32, device=DEV) for _ in range(2)]
    H, lse, am = _outs(R)
    for l in range(n):
        idx = None if l == 0 else act[(l - 1) & 1]
        c = None if l == 0 else cnt[(l - 1) & 1]
        B.eh_eval(ctx, l, hid.h[l], R, H, lse, am, row_idx=idx, n_rows_dev=c)
        B.eh_exit_decide(ctx, l, H, am, R, ex2, tok2, act[l & 1], cnt[l & 1], row_idx=idx, n_rows_dev=c)
        torch.cuda.synchronize()
        live = cnt[l & 1].item()
        expect = [r for r in range(R) if ex2[r].item() < 0]
        assert act[l & 1][:live].tolist() == expect          # stable compaction
    assert torch.equal(ex, ex2) and torch.equal(tok, tok2)
    B.eh_destroy(ctx)


def test_nan_row_is_defined_behaviour(B):
    w = G.Workload("nan", d=64, V=300, n_heads=2, rows=4, dtype="f32", seed=23)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    hid.h[0, 2, 5] = float("nan")
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [100.0, float("inf")], max_rows=4)
    ex = torch.full((4,), -1, dtype=torch.int32, device=DEV)
    tok = torch.full((4,), -1, dtype=torch.int32, device=DEV)
    Hout = torch.zeros((2, 4), device=DEV)
    B.eh_cascade(ctx, hid.h, 4, ex, tok, Hout, None)
    torch.cuda.synchronize()
    assert math.isnan(Hout[0, 2].item())
    assert ex.tolist() == [0, 0, 1, 0]          # NaN never passes the test; falls to the final head
    B.eh_destroy(ctx)


def test_eval_heads_equals_eval_per_head(B):
    """The many-heads entry point against the oracle on one head and, bit for bit, against
    eh_eval on every head (same kernels on the same data); also its one-head-at-a-time
    fallback (fp32, and bf16 with at most 16 rows) and a second, smaller call on the same
    context (the workspace is reused)."""
    for dtype, rows in (("bf16", 100), ("bf16", 37), ("bf16", 9), ("f32", 40)):
        w = G.scaled(G.CONFIGS["c2_calib"], d=256, V=3000, n_heads=4, rows=rows, dtype=dtype)
        heads = G.make_heads(w, DEV)
        hid = G.make_hidden(w, heads, DEV)
        ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=100)
        n = 3
        H = torch.full((n, rows), float("nan"), device=DEV)
        lse = torch.full((n, rows), float("nan"), device=DEV)
        am = torch.full((n, rows), -1, dtype=torch.int32, device=DEV)
        B.eh_eval_heads(ctx, 1, n, hid.h[1:], rows, H, lse, am)
        torch.cuda.synchronize()
        for l in range(n):
            H1, l1, a1 = _outs(rows)
            B.eh_eval(ctx, 1 + l, hid.h[1 + l], rows, H1, l1, a1)
            torch.cuda.synchronize()
            assert torch.equal(H[l], H1) and torch.equal(lse[l], l1) and torch.equal(am[l], a1), (dtype, rows, l)
        orc = P.oracle_head(hid.h[2], heads.gamma[2], heads.beta[2], heads.W[2], dtype == "bf16")
        P.compare_head(f"heads/{dtype}/{rows}", H[1], lse[1], am[1], orc, [])
        B.eh_destroy(ctx)


def test_determinism(B):
    w = G.scaled(G.CONFIGS["c1_decode"], n_heads=2, rows=8)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=8)
    ref = None
    for _ in range(20):
        H, lse, am = _outs(8)
        B.eh_eval(ctx, 1, hid.h[1], 8, H, lse, am)
        torch.cuda.synchronize()
        cur = (H.clone(), lse.clone(), am.clone())
        if ref is not None:
            assert all(torch.equal(a, b) for a, b in zip(ref, cur))
        ref = cur
    B.eh_destroy(ctx)


# --------------------------------------------------------------- config 0
def test_c0_tiny_full(B):
    w = G.CONFIGS["c0_tiny"]
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    tau = G.tau_linear(w)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=w.rows)
    log = []
    _eval_all(B, ctx, heads, hid, w.rows, False, "c0", log)
    full = P.oracle_all_heads(heads, hid.h, False)
    ex = torch.full((w.rows,), -1, dtype=torch.int32, device=DEV)
    tok = torch.full((w.rows,), -1, dtype=torch.int32, device=DEV)
    Hout = torch.zeros((w.n_heads, w.rows), device=DEV)
    B.eh_cascade(ctx, hid.h, w.rows, ex, tok, Hout, None)
    torch.cuda.synchronize()
    P.compare_cascade("c0", ex, tok, Hout, full[0], full[2], full[3], tau, log)
    print("c0 exit layers:", ex.tolist(), "near-ties:", log)
    B.eh_destroy(ctx)


# --------------------------------------------------------------- config 1
@pytest.mark.timeout(900)
def test_c1_decode_steps(B):
    """Batch-1 cascades over 2048 seeded decode steps, every one of them checked against the
    oracle (every head on every step: exit layer, token, and the entropy of each head up to
    the exit)."""
    w = G.CONFIGS["c1_decode"]
    heads = G.make_heads(w, DEV)
    steps = w.steps
    hid = G.make_hidden(w, heads, DEV, rows=steps)        # [24, 2048, 1024]: row t = decode step t
    tau = G.tau_linear(w)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=1)
    ex = torch.full((steps,), -1, dtype=torch.int32, device=DEV)
    tok = torch.full((steps,), -1, dtype=torch.int32, device=DEV)
    Hout = torch.zeros((steps, w.n_heads), device=DEV)
    nev = torch.zeros(1, dtype=torch.int64, device=DEV)
    for t in range(steps):
        B.eh_cascade(ctx, hid.h[:, t:t + 1], 1, ex[t:t + 1], tok[t:t + 1], Hout[t], nev)
    torch.cuda.synchronize()
    assert ((ex >= 0) & (ex < w.n_heads)).all() and ((tok >= 0) & (tok < w.V)).all()
    assert int(nev.item()) == int((ex.long() + 1).sum().item())
    full = P.oracle_all_heads(heads, hid.h, True)
    log = []
    flips = P.compare_cascade("c1", ex, tok, Hout.T.contiguous(), full[0], full[2], full[3], tau, log)
    print(f"c1: mean evals/step {nev.item() / steps:.2f}; all {steps} steps checked; flips {flips}; log {log}")
    assert len(set(ex.tolist())) >= 8          # exits are spread over many depths
    B.eh_destroy(ctx)


# --------------------------------------------------------------- config 2
def test_c2_batched_calibration(B):
    """All 24 heads on all 512 tokens; the oracle checks every head on 64
    sampled tokens and three heads on all 512."""
    w = G.CONFIGS["c2_calib"]
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    R = w.rows
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=R)
    sample = torch.arange(0, R, 8, device=DEV)
    log = []
    per_head = []
    for l in range(w.n_heads):
        H, lse, am = _outs(R)
        B.eh_eval(ctx, l, hid.h[l], R, H, lse, am)
        torch.cuda.synchronize()
        per_head.append((H, lse, am))
        sel = slice(None) if l in (0, 11, 23) else sample
        orc = P.oracle_head(hid.h[l][sel], heads.gamma[l], heads.beta[l], heads.W[l], True)
        P.compare_head(f"c2/head{l}", H[sel], lse[sel], am[sel], orc, log)
    print("c2 near-ties:", log)
    # the form bench.py times: all heads in one call (one projection launch for the 24 heads),
    # bit for bit what the per-head calls gave; then the same with the two extra metrics
    Hb = torch.full((w.n_heads, R), float("nan"), device=DEV)
    Lb = torch.full((w.n_heads, R), float("nan"), device=DEV)
    Ab = torch.full((w.n_heads, R), -7, dtype=torch.int32, device=DEV)
    B.eh_eval_heads(ctx, 0, w.n_heads, hid.h, R, Hb, Lb, Ab)
    torch.cuda.synchronize()
    for l in range(w.n_heads):
        assert torch.equal(Hb[l], per_head[l][0]) and torch.equal(Lb[l], per_head[l][1])
        assert torch.equal(Ab[l], per_head[l][2])
    for _ in range(3):                                        # and the same bits on every repeat
        Hr, Lr, Ar = torch.zeros_like(Hb), torch.zeros_like(Lb), torch.zeros_like(Ab)
        B.eh_eval_heads(ctx, 0, w.n_heads, hid.h, R, Hr, Lr, Ar)
        torch.cuda.synchronize()
        assert torch.equal(Hr, Hb) and torch.equal(Lr, Lb) and torch.equal(Ar, Ab)
    Pm = torch.full((w.n_heads, R), float("nan"), device=DEV)
    Mg = torch.full((w.n_heads, R), float("nan"), device=DEV)
    H2, L2, A2 = torch.zeros_like(Hb), torch.zeros_like(Lb), torch.zeros_like(Ab)
    B.eh_eval_heads_metrics(ctx, 0, w.n_heads, hid.h, R, H2, L2, A2, Pm, Mg)
    torch.cuda.synchronize()
    assert torch.equal(H2, Hb) and torch.equal(L2, Lb) and torch.equal(A2, Ab)
    for l in (3, 20):
        sel = sample[:32]
        pm_o, mg_o = O.head_metrics(P.f64(hid.h[l][sel]), P.f64(heads.gamma[l]), P.f64(heads.beta[l]),
                                    P.f64(heads.W[l]), 1e-5, True)
        dp = np.abs(Pm[l][sel].double().cpu().numpy() - pm_o).max()
        dm = np.abs(Mg[l][sel].double().cpu().numpy() - mg_o).max()
        assert dp <= TOL_P and dm <= TOL_P, (l, dp, dm)
    B.eh_destroy(ctx)


# --------------------------------------------------------------- configs 3, 4
@pytest.fixture(scope="module")
def big(B):
    """The 32 Pythia-2.8B-shaped heads shared by configs 3 and 4, with the
    oracle's statistics of every head on config 3's 64 rows and on the
    16 x 8 drafting rows of config 4."""
    w3 = G.CONFIGS["c3_dynexit"]
    heads = G.make_heads(w3, DEV)
    hid3 = G.make_hidden(w3, heads, DEV)
    hid4 = G.make_hidden(w3, heads, DEV, rows=16 * 8, seed_offset=404)
    outs3, outs4 = [], []
    for l in range(w3.n_heads):
        W64 = P.f64(heads.W[l])
        both = torch.cat([hid3.h[l], hid4.h[l]])
        o = P.oracle_head(both, heads.gamma[l], heads.beta[l], None, True, W64=W64)
        outs3.append([x[:64] for x in o])
        outs4.append([x[64:] for x in o])
        del W64
    st = lambda outs, i: np.stack([o[i] for o in outs])
    full3 = tuple(st(outs3, i) for i in range(4))
    full4 = tuple(st(outs4, i) for i in range(4))
    return dict(w=w3, heads=heads, hid3=hid3, hid4=hid4, full3=full3, full4=full4)


def test_c3_dynamic_exit_with_compaction(B, big):
    w, heads, hid, full = big["w"], big["heads"], big["hid3"], big["full3"]
    tau = G.tau_for_schedule(full[0], w.n_heads)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=w.rows)
    R = w.rows
    ex = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    tok = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    Hout = torch.zeros((w.n_heads, R), device=DEV)
    nev = torch.zeros(1, dtype=torch.int64, device=DEV)
    B.eh_cascade(ctx, hid.h, R, ex, tok, Hout, nev)
    torch.cuda.synchronize()
    log = []
    P.compare_cascade("c3", ex, tok, Hout, full[0], full[2], full[3], tau, log)
    exl = ex.cpu().numpy()
    frac = [(exl < l).mean() for l in (8, 16, 24)]
    print(f"c3 exited fraction by layers 8/16/24: {frac}; evals {nev.item()}; log {log}")
    # run to run the results are the same bits (the next head's row list is filled in arrival order,
    # which must not show in any output)
    for _ in range(3):
        ex2 = torch.full((R,), -1, dtype=torch.int32, device=DEV)
        tok2 = torch.full((R,), -1, dtype=torch.int32, device=DEV)
        Hout2 = torch.zeros((w.n_heads, R), device=DEV)
        B.eh_cascade(ctx, hid.h, R, ex2, tok2, Hout2, None)
        torch.cuda.synchronize()
        assert torch.equal(ex, ex2) and torch.equal(tok, tok2)
        assert torch.equal(Hout.view(torch.int32), Hout2.view(torch.int32))
    assert abs(frac[0] - 0.10) < 0.05 and abs(frac[1] - 0.40) < 0.05 and abs(frac[2] - 0.70) < 0.05
    big["tau3"] = tau
    B.eh_destroy(ctx)


def test_c4_dssd_verify(B, big):
    w, heads, full4 = big["w"], big["heads"], big["full4"]
    Bsz, k = 16, 8
    tau = big.get("tau3") or G.tau_for_schedule(big["full3"][0], w.n_heads)
    # drafts = the oracle's argmax at each drafting row's dynamic exit layer
    draft = np.empty(Bsz * k, dtype=np.int64)
    for r in range(Bsz * k):
        e = O.exit_rule(full4[0][:, r], tau)
        draft[r] = full4[2][e, r]
    draft_t = torch.from_numpy(draft.reshape(Bsz, k)).to(DEV)
    case = G.make_verify_case(w, heads, draft_t, DEV)
    fin = w.n_heads - 1
    acc_o, nxt_o, tgt_o, gap_o = O.dssd_verify(
        P.f64(case.f_final), draft.reshape(Bsz, k), P.f64(heads.gamma[fin]), P.f64(heads.beta[fin]),
        P.f64(heads.W[fin]), None, 1e-5, True)
    assert gap_o.min() > 1e-2, "verification inputs must decide clearly"
    ctx = B.eh_create(heads.W[fin:], heads.gamma[fin:], heads.beta[fin:], [float("inf")], max_rows=Bsz * (k + 1))
    acc = torch.full((Bsz,), -1, dtype=torch.int32, device=DEV)
    nxt = torch.full((Bsz,), -1, dtype=torch.int32, device=DEV)
    tgt = torch.full((Bsz, k + 1), -1, dtype=torch.int32, device=DEV)
    d32 = draft_t.to(torch.int32).contiguous()
    B.dssd_verify(ctx, case.f_final, d32, None, acc, nxt, tgt)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tgt.cpu().numpy(), tgt_o)
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), nxt_o)
    # truncated drafts
    dl = torch.tensor([0, 1, 2, 3, 4, 5, 6, 7, 8, 8, 3, 0, 8, 2, 5, 1], dtype=torch.int32, device=DEV)
    B.dssd_verify(ctx, case.f_final, d32, dl, acc, nxt, None)
    torch.cuda.synchronize()
    acc_t, nxt_t, _, _ = O.dssd_verify(
        P.f64(case.f_final), draft.reshape(Bsz, k), P.f64(heads.gamma[fin]), P.f64(heads.beta[fin]),
        P.f64(heads.W[fin]), dl.cpu().numpy(), 1e-5, True)
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_t)
    np.testing.assert_array_equal(nxt.cpu().numpy(), nxt_t)
    print(f"c4: accepted {acc_o.tolist()} mean {acc_o.mean():.2f}; agreement {case.agree[:, :k].float().mean().item():.2f}")
    B.eh_destroy(ctx)


# --------------------------------------------------------------- threshold calibration
EPS_SWEEP = [0.5, 0.55, 0.6, 0.65, 0.7, 0.75, 0.8, 0.85, 0.9, 0.95, 1.0]


def _calibrate(B, ctx, H, pred, ref, eps):
    tau = torch.full((len(eps),), float("nan"), device=DEV)
    n = torch.full((len(eps),), -1, dtype=torch.int64, device=DEV)
    B.eh_calibrate(ctx, H, pred, ref, eps, tau, n)
    torch.cuda.synchronize()
    return tau.cpu().numpy(), n.cpu().numpy()


@pytest.fixture(scope="module")
def small_ctx(B):
    w = G.Workload("calib", d=64, V=64, n_heads=1, rows=4, dtype="bf16", seed=1)
    heads = G.make_heads(w, DEV)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [float("inf")], max_rows=4)
    yield ctx
    B.eh_destroy(ctx)


@pytest.mark.parametrize("M,ties,nan_every", [(1, False, 0), (2, True, 0), (257, False, 0), (1000, True, 0),
                                              (2500, False, 7), (3000, True, 5)])
def test_calibrate_matches_oracle(B, small_ctx, M, ties, nan_every):
    """Bit-exact: the threshold is one of the input entropies and the count is an integer."""
    H, pred, ref = G.make_calibration_case(M, DEV, seed=M, V=50, ties=ties, nan_every=nan_every)
    eps = [0.0, 0.01] + EPS_SWEEP
    tau, n = _calibrate(B, small_ctx, H, pred, ref, eps)
    Hc = H.cpu().numpy().astype(np.float64)
    t = O.correctness(pred.cpu().numpy(), ref.cpu().numpy())
    for i, e in enumerate(eps):
        want_tau, want_n = O.calibrate_threshold(Hc, t, e)
        assert (tau[i] == np.float32(want_tau)) and int(n[i]) == want_n, (M, e, tau[i], want_tau, n[i], want_n)


@pytest.mark.parametrize("M,ties,nan_every", [(257, False, 0), (3000, True, 5), (40000, False, 11)])
def test_calibrate_by_sorting_gives_the_same(B, small_ctx, M, ties, nan_every, monkeypatch):
    """eh_calibrate has two ways to the same answer: counting in three levels of bins, and,
    for data whose proportion hovers at a level over many bins, a full sort.  The sort is
    forced here (the library reads EH_CALIBRATE_SORT at every call) and held to the oracle,
    and to what the call returns without it, bit for bit."""
    H, pred, ref = G.make_calibration_case(M, DEV, seed=M + 1, V=50, ties=ties, nan_every=nan_every)
    eps = [0.0, 0.01] + EPS_SWEEP
    before = B.eh_probe_calibrate_sorted(small_ctx)
    tau, n = _calibrate(B, small_ctx, H, pred, ref, eps)
    mid = B.eh_probe_calibrate_sorted(small_ctx)
    monkeypatch.setenv("EH_CALIBRATE_SORT", "1")
    tau_s, n_s = _calibrate(B, small_ctx, H, pred, ref, eps)
    monkeypatch.delenv("EH_CALIBRATE_SORT")
    assert B.eh_probe_calibrate_sorted(small_ctx) == mid + 1 and mid - before in (0, 1)
    np.testing.assert_array_equal(tau, tau_s)
    np.testing.assert_array_equal(n, n_s)
    if M <= 3000:
        Hc = H.cpu().numpy().astype(np.float64)
        t = O.correctness(pred.cpu().numpy(), ref.cpu().numpy())
        for i, e in enumerate(eps):
            want_tau, want_n = O.calibrate_threshold(Hc, t, e)
            assert (tau_s[i] == np.float32(want_tau)) and int(n_s[i]) == want_n, (M, e, tau_s[i], want_tau)


def _calibrate_by_counting(H, t, eps):
    """The definition by exact counting (tokens and correct tokens at or below every distinct
    entropy value, from sorted arrays): the unique answer for every level, at any size."""
    ok = ~np.isnan(H)
    vals, inv = np.unique(H[ok], return_inverse=True)                      # ascending entropy values
    cnt = np.bincount(inv, minlength=len(vals)).cumsum()                   # tokens with H <= value
    cor = np.bincount(inv, weights=t[ok], minlength=len(vals)).cumsum()    # correct ones among them
    out = []
    for e in eps:
        good = cor / cnt >= e                                              # the section's quotient, in double
        if not good.any():
            out.append((-np.inf, 0))
        else:
            k = np.nonzero(good)[0].max()                                  # largest qualifying value
            out.append((np.float32(vals[k]), int(cnt[k])))
    return out


@pytest.mark.parametrize("spread", ["uniform", "one_binade", "wide"])
def test_calibrate_hovering_proportion(B, small_ctx, spread):
    """Predictions that are right half of the time whatever the entropy: at the level 0.5 the
    proportion stays within a hair of the level over the whole range of thresholds, which is
    what the counting refinement cannot prune.  The call must still return the exact answer
    (the full sort serves it), and levels away from 0.5 must not need the sort."""
    M = 1 << 18
    gen = torch.Generator(device=DEV).manual_seed(77)
    u = torch.rand(M, generator=gen, device=DEV)
    if spread == "uniform":
        H = u * 8.0
    elif spread == "one_binade":
        H = 4.0 + u * 3.9
    else:
        H = torch.exp(u * 60.0 - 50.0)
    H = H.to(torch.float32).contiguous()
    ref = torch.zeros(M, dtype=torch.int32, device=DEV)
    pred = (torch.rand(M, generator=gen, device=DEV) < 0.5).to(torch.int32)
    Hc = H.cpu().numpy().astype(np.float64)
    t = O.correctness(pred.cpu().numpy(), ref.cpu().numpy())
    for eps, may_sort in (([0.5, 0.4999, 0.5001], True), ([0.3, 0.45, 0.55, 0.9, 1.0], False)):
        before = B.eh_probe_calibrate_sorted(small_ctx)
        tau, n = _calibrate(B, small_ctx, H, pred, ref, eps)
        sorted_calls = B.eh_probe_calibrate_sorted(small_ctx) - before
        assert may_sort or sorted_calls == 0, (spread, eps)
        for i, (want_tau, want_n) in enumerate(_calibrate_by_counting(Hc, t, eps)):
            assert tau[i] == want_tau and n[i] == want_n, (spread, eps[i], tau[i], want_tau, n[i], want_n)


def test_calibrate_degenerate_inputs(B, small_ctx):
    H = torch.tensor([0.5, 0.25, 2.0, 0.0, -0.0], device=DEV)
    same = torch.zeros(5, dtype=torch.int32, device=DEV)
    tau, n = _calibrate(B, small_ctx, H, same, same, [0.0, 1.0])          # all right
    assert list(tau) == [2.0, 2.0] and list(n) == [5, 5]
    tau, n = _calibrate(B, small_ctx, H, same, same + 1, [0.0, 0.5, 1.0])  # all wrong
    assert tau[0] == 2.0 and n[0] == 5 and np.isneginf(tau[1:]).all() and list(n[1:]) == [0, 0]
    right_at_zero = torch.tensor([1, 1, 1, 0, 0], dtype=torch.int32, device=DEV)
    tau, n = _calibrate(B, small_ctx, H, same, right_at_zero, [1.0])       # +0 and -0 are one value
    assert tau[0] == 0.0 and n[0] == 2
    allnan = torch.full((9,), float("nan"), device=DEV)
    nine = torch.zeros(9, dtype=torch.int32, device=DEV)
    tau, n = _calibrate(B, small_ctx, allnan, nine, nine, [0.0, 0.5])
    assert np.isneginf(tau).all() and list(n) == [0, 0]
    tau, n = _calibrate(B, small_ctx, H[:0], same[:0], same[:0], [0.3])    # empty set
    assert np.isneginf(tau).all() and list(n) == [0]


@pytest.mark.parametrize("ties", [True, False])
def test_calibrate_large_set_properties(B, small_ctx, ties):
    """2^22 tokens, beyond what the quadratic oracle can do: the definition is evaluated by
    exact counting instead, with tied entropies and without."""
    M = 1 << 22
    H, pred, ref = G.make_calibration_case(M, DEV, seed=3, ties=ties, nan_every=1001)
    before = B.eh_probe_calibrate_sorted(small_ctx)
    tau, n = _calibrate(B, small_ctx, H, pred, ref, EPS_SWEEP)
    assert B.eh_probe_calibrate_sorted(small_ctx) == before, "data of this kind must not need the full sort"
    Hc = H.cpu().numpy().astype(np.float64)
    t = O.correctness(pred.cpu().numpy(), ref.cpu().numpy())
    for i, (want_tau, want_n) in enumerate(_calibrate_by_counting(Hc, t, EPS_SWEEP)):
        assert tau[i] == want_tau and n[i] == want_n, (EPS_SWEEP[i], tau[i], want_tau, n[i], want_n)
    assert (np.diff(tau) <= 0).all()


# --------------------------------------------------------------- the other two confidence metrics
@pytest.mark.parametrize("V,d,R", [(1000, 128, 5), (777, 512, 37), (3000, 256, 161), (1500, 160, 700), (1, 64, 3)])
def test_eval_heads_metrics(B, V, d, R):
    w = G.Workload("metrics", d=d, V=V, n_heads=3, rows=R, dtype="bf16", seed=V + d + R)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=R)
    n = 3
    H = torch.full((n, R), float("nan"), device=DEV)
    lse = torch.full((n, R), float("nan"), device=DEV)
    am = torch.full((n, R), -1, dtype=torch.int32, device=DEV)
    pm = torch.full((n, R), float("nan"), device=DEV)
    mg = torch.full((n, R), float("nan"), device=DEV)
    B.eh_eval_heads_metrics(ctx, 0, n, hid.h, R, H, lse, am, pm, mg)
    torch.cuda.synchronize()
    f64 = G.to_f64_numpy
    for l in range(n):
        orc = P.oracle_head(hid.h[l], heads.gamma[l], heads.beta[l], heads.W[l], True)
        P.compare_head(f"metrics/head{l}", H[l], lse[l], am[l], orc, [])
        pm_o, mg_o = O.head_metrics(f64(hid.h[l]), f64(heads.gamma[l]), f64(heads.beta[l]), f64(heads.W[l]),
                                    1e-5, True)
        dp = np.abs(pm[l].double().cpu().numpy() - pm_o).max()
        dm = np.abs(mg[l].double().cpu().numpy() - mg_o).max()
        assert dp <= TOL_P and dm <= TOL_P, (l, dp, dm)
    if R > 16:   # the statistics are those of eh_eval_heads, bit for bit
        H2 = torch.zeros_like(H)
        l2 = torch.zeros_like(lse)
        a2 = torch.zeros_like(am)
        B.eh_eval_heads(ctx, 0, n, hid.h, R, H2, l2, a2)
        torch.cuda.synchronize()
        assert torch.equal(H, H2) and torch.equal(lse, l2) and torch.equal(am, a2)
    B.eh_destroy(ctx)


def test_eval_heads_metrics_tie_at_the_top_and_refusals(B):
    # two identical vocabulary rows that win: the margin is exactly 0
    w = G.Workload("tie", d=64, V=200, n_heads=1, rows=40, dtype="bf16", seed=5)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    f64 = G.to_f64_numpy
    z = O.head_logits(O.layernorm(f64(hid.h[0]), f64(heads.gamma[0]), f64(heads.beta[0]), 1e-5, True), f64(heads.W[0]))
    win = int(np.bincount(z.argmax(axis=1)).argmax())           # the most frequent winner
    Wt = heads.W[0].clone()
    Wt[(win + 97) % 200] = Wt[win]
    ctx = B.eh_create([Wt], heads.gamma, heads.beta, [float("inf")], max_rows=40)
    pm = torch.zeros((1, 40), device=DEV)
    mg = torch.ones((1, 40), device=DEV)
    am = torch.zeros((1, 40), dtype=torch.int32, device=DEV)
    B.eh_eval_heads_metrics(ctx, 0, 1, hid.h, 40, None, None, am, pm, mg)
    torch.cuda.synchronize()
    rows = np.nonzero(z.argmax(axis=1) == win)[0]
    assert len(rows) > 0 and (mg[0, rows] == 0).all() and (am[0, rows].cpu().numpy() == min(win, (win + 97) % 200)).all()
    B.eh_destroy(ctx)
    w32 = G.scaled(w, dtype="f32")
    h32 = G.make_heads(w32, DEV)
    ctx = B.eh_create(h32.W, h32.gamma, h32.beta, [float("inf")], max_rows=40)
    with pytest.raises(B.EhError):
        B.eh_eval_heads_metrics(ctx, 0, 1, G.make_hidden(w32, h32, DEV).h, 40, None, None, None, pm, mg)
    B.eh_destroy(ctx)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("Bsz,k", [(5, 4), (3, 2), (7, 9), (9, 16), (4, 49), (8, 31), (2, 127), (40, 5)])
def test_dssd_verify_small(B, dtype, Bsz, k):
    """Verification on small shapes: with and without draft lengths, with and without the
    target output, through the decode kernel (at most 16 positions), the persistent kernel for up
    to 256 positions (1 to 8 blocks of 32; a draft longer than one wave's 64 positions; more draft
    rows than a wave) and the batched one (fp32)."""
    w = G.Workload("verify", d=128, V=900, n_heads=2, rows=Bsz * (k + 1), dtype=dtype, seed=Bsz * 10 + k)
    heads = G.make_heads(w, DEV)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(k)
    draft = torch.randint(0, w.V, (Bsz, k), generator=gen).to(DEV)
    case = G.make_verify_case(w, heads, draft, DEV)
    dlen = torch.randint(0, k + 1, (Bsz,), generator=gen).to(torch.int32).to(DEV)
    fin = w.n_heads - 1
    f64 = G.to_f64_numpy
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [0.0, float("inf")], max_rows=Bsz * (k + 1))
    for use_len in (False, True):
        acc_o, nxt_o, tgt_o, gap_o = O.dssd_verify(f64(case.f_final), draft.cpu().numpy(), f64(heads.gamma[fin]),
                                                   f64(heads.beta[fin]), f64(heads.W[fin]),
                                                   dlen.cpu().numpy() if use_len else None, 1e-5, dtype == "bf16")
        assert gap_o.min() > 1e-3
        acc = torch.full((Bsz,), -1, dtype=torch.int32, device=DEV)
        nxt = torch.full((Bsz,), -1, dtype=torch.int32, device=DEV)
        tgt = torch.full((Bsz, k + 1), -1, dtype=torch.int32, device=DEV)
        B.dssd_verify(ctx, case.f_final, draft.to(torch.int32).contiguous(), dlen if use_len else None, acc, nxt,
                      tgt if use_len else None)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
        np.testing.assert_array_equal(nxt.cpu().numpy(), nxt_o)
        if use_len:
            np.testing.assert_array_equal(tgt.cpu().numpy(), tgt_o)
    B.eh_destroy(ctx)


# --------------------------------------------------------------- DSSD drafting phase
def _draft_case(dtype, seed, n_heads=4, n_pos=12, V=1000, d=256, kappa=0.25):
    """A seeded drafting case whose oracle argmaxes are all clear of a tie (top-2 logit gap above
    1e-3): the first seed from `seed` on that has none, so the comparison can be exact."""
    for s in range(seed, seed + 16):
        w = G.Workload("draft", d=d, V=V, n_heads=n_heads, rows=n_pos, dtype=dtype, seed=s, kappa=kappa)
        heads = G.make_heads(w, DEV)
        hid = G.make_hidden(w, heads, DEV)                  # [n_heads, n_pos, d]
        full = P.oracle_all_heads(heads, hid.h, dtype == "bf16")
        if full[3].min() > 1e-3:
            return w, heads, hid, full
    raise AssertionError("no tie-free case in 16 seeds")


def _run_draft(B, heads, hid, tau, limit, eos, n_pos=None):
    """One dssd_draft call; every output starts poisoned."""
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=1)
    hp = hid.h.permute(1, 0, 2)                             # [position, head, d], a strided view
    if n_pos is not None:
        hp = hp[:n_pos]
    draft = torch.full((max(limit, 1),), -7, dtype=torch.int32, device=DEV)
    layers = torch.full((max(limit, 1),), -7, dtype=torch.int32, device=DEV)
    ln = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    reason = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    fb = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    nev = torch.zeros(1, dtype=torch.int64, device=DEV)
    B.dssd_draft(ctx, hp, limit, eos, draft, ln, layers, reason, fb, nev)
    torch.cuda.synchronize()
    B.eh_check(ctx)
    B.eh_destroy(ctx)
    n = int(ln.item())
    return dict(draft=draft[:n].tolist(), exit_layer=layers[:n].tolist(), reason=B.DRAFT_REASONS[int(reason.item())],
                fallback_token=int(fb.item()), n_evals=int(nev.item())), layers.tolist()


def _safe_tau(H, q, margin=5e-3):
    """Per-head thresholds near the q-quantile of the oracle's entropies, moved into the widest
    gap nearby so that no entropy lies within `margin` of its head's threshold."""
    tau = []
    for l in range(H.shape[0]):
        s = np.sort(H[l])
        k = min(max(int(q * len(s)), 1), len(s) - 1)
        best = max(range(max(1, k - 3), min(len(s), k + 4)), key=lambda i: s[i] - s[i - 1])
        assert s[best] - s[best - 1] > 2 * margin
        tau.append(float(0.5 * (s[best] + s[best - 1])))
    return tau


@pytest.mark.parametrize("dtype,d", [("bf16", 256), ("f32", 256), ("bf16", 2176)])
def test_dssd_draft_matches_oracle(B, dtype, d):
    """d = 2176 is beyond the single-row kernel: the positions' cascades then run the persistent
    kernel for up to 256 rows, with the same controller behind each."""
    # the planted direction's pull grows with sqrt(d): scaled back so that the entropies spread as at d = 256
    w, heads, hid, (H, _, am, gap) = _draft_case(dtype, seed=2024, d=d, kappa=0.25 * math.sqrt(256 / d))
    Ht, amt = H.T, am.T                                     # [position][head]
    n_heads, n_pos = H.shape
    seen = set()
    for q in (0.3, 0.6, 0.85):
        tau = _safe_tau(H, q)
        for limit in (3, 8, 12, 20):
            want = O.dssd_draft(Ht, amt, tau, limit, -1)
            got, layers = _run_draft(B, heads, hid, tau, limit, -1)
            assert got == want, (q, limit, got, want)
            assert all(x == -1 for x in layers[len(want["draft"]):limit])
            seen.add(want["reason"])
            if want["draft"]:
                # the same call with its own last drafted token as the end-of-sequence token
                eos = want["draft"][-1]
                want_e = O.dssd_draft(Ht, amt, tau, limit, eos)
                got_e, _ = _run_draft(B, heads, hid, tau, limit, eos)
                assert got_e == want_e and want_e["reason"] == "eos"
                seen.add("eos")
    assert {"limit", "fallback", "eos"} <= seen, seen
    # every exit head always confident: the buffer fills, or the positions run out
    always = [1e9] * n_heads
    for limit, npos in ((5, None), (12, None), (20, None), (8, 4), (8, 0), (0, None)):
        hsel = Ht if npos is None else Ht[:npos]
        want = O.dssd_draft(hsel, amt, always, limit, -1)
        got, _ = _run_draft(B, heads, hid, always, limit, -1, n_pos=npos)
        assert got == want, (limit, npos, got, want)
        seen.add(want["reason"])
    assert "exhausted" in seen
    # no exit head ever confident: the model's head answers at the first position
    never = [-1.0] * n_heads
    want = O.dssd_draft(Ht, amt, never, 8, -1)
    got, _ = _run_draft(B, heads, hid, never, 8, -1)
    assert got == want and want["reason"] == "fallback" and want["n_evals"] == n_heads and want["draft"] == []


def test_dssd_draft_errors(B):
    w, heads, hid, _ = _draft_case("bf16", seed=7, n_heads=2, n_pos=2, V=64, d=64)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [1.0, 1.0], max_rows=1)
    i32 = lambda n: torch.zeros(n, dtype=torch.int32, device=DEV)
    with pytest.raises(B.EhError):
        B.dssd_draft(ctx, hid.h.permute(1, 0, 2), -1, -1, i32(4), i32(1), i32(4))
    with pytest.raises(B.EhError):
        B.dssd_draft(ctx, hid.h.permute(1, 0, 2), 4, -1, None, i32(1), i32(4))
    B.eh_destroy(ctx)
    # a context with a bias vector has no single-row kernel: drafting is refused, not emulated
    bias = [torch.zeros(64, device=DEV) for _ in heads.W]
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, [1.0, 1.0], max_rows=1, bias=bias)
    with pytest.raises(B.EhError):
        B.dssd_draft(ctx, hid.h.permute(1, 0, 2), 4, -1, i32(4), i32(1), i32(4))
    B.eh_destroy(ctx)


# --------------------------------------------------------------- verification bookkeeping
def test_dssd_tally_matches_oracle(B, small_ctx):
    rng = np.random.default_rng(77)
    counters = torch.zeros(5, dtype=torch.int64, device=DEV)
    total = dict(rounds=0, drafted=0, accepted=0, wasted=0, exit_layer_sum=0)
    for Bsz, k, with_len, with_layers in ((1, 1, True, True), (16, 8, True, True), (1000, 32, True, True),
                                          (300, 5, False, True), (77, 9, True, False), (64, 0, True, True)):
        lens = rng.integers(0, k + 1, size=Bsz)
        acc = np.array([rng.integers(0, n + 1) for n in (lens if with_len else np.full(Bsz, k))])
        layers = rng.integers(0, 24, size=(Bsz, max(k, 1)))[:, :k]
        want = O.dssd_tally(lens if with_len else np.full(Bsz, k), acc, layers if with_layers else None)
        for key in total:
            total[key] += want[key]
        B.dssd_tally(small_ctx, torch.tensor(lens, dtype=torch.int32, device=DEV) if with_len else None,
                     torch.tensor(acc, dtype=torch.int32, device=DEV), Bsz, k,
                     torch.tensor(layers, dtype=torch.int32, device=DEV).contiguous() if with_layers else None,
                     counters)
        torch.cuda.synchronize()
        assert counters.tolist() == [total[x] for x in ("rounds", "drafted", "accepted", "wasted", "exit_layer_sum")]
    # zero rounds change nothing; values outside their range are clamped (length to [0, k], accepted to [0, length])
    before = counters.tolist()
    B.dssd_tally(small_ctx, None, torch.zeros(1, dtype=torch.int32, device=DEV), 0, 4, None, counters)
    torch.cuda.synchronize()
    assert counters.tolist() == before
    B.dssd_tally(small_ctx, torch.tensor([9, -3, 2], dtype=torch.int32, device=DEV),
                 torch.tensor([7, 1, -1], dtype=torch.int32, device=DEV), 3, 4, None, counters)
    torch.cuda.synchronize()
    want = O.dssd_tally([4, 0, 2], [4, 0, 0])
    assert counters.tolist() == [before[0] + 3, before[1] + want["drafted"], before[2] + want["accepted"],
                                 before[3] + want["wasted"], before[4]]
    with pytest.raises(B.EhError):
        B.dssd_tally(small_ctx, None, torch.zeros(1, dtype=torch.int32, device=DEV), 1, 4, None, None)


# --------------------------------------------------------------- training objectives (Section 3.3)
TOL_LOSS_ABS, TOL_LOSS_REL = 2e-3, 1e-4     # as for the entropy: fp32 logits, one exponential per logit


def _loss_case(V, d, R, seed):
    w = G.Workload("loss", d=d, V=V, n_heads=3, rows=R, dtype="bf16", seed=seed)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed + 5)
    labels = torch.randint(0, V, (R,), generator=gen, device=DEV, dtype=torch.int32)
    return w, heads, hid, labels


def _oracle_losses(heads, hid, head, labels, alpha):
    f = P.f64
    fin = len(heads.W) - 1
    return O.head_losses(f(hid.h[head]), f(hid.h[fin]), f(heads.gamma[head]), f(heads.beta[head]), f(heads.W[head]),
                         f(heads.gamma[fin]), f(heads.beta[fin]), f(heads.W[fin]),
                         None if labels is None else labels.cpu().numpy(), alpha, 1e-5, True)


def _close(got, want):
    return np.abs(got - want) <= TOL_LOSS_ABS + TOL_LOSS_REL * np.abs(want)


@pytest.mark.parametrize("V,d,R", [(1000, 256, 5), (777, 512, 37), (2048, 256, 161), (1500, 160, 300), (33, 64, 33),
                                   (4096, 128, 128), (50, 32, 1)])
def test_head_losses_match_oracle(B, V, d, R):
    w, heads, hid, labels = _loss_case(V, d, R, seed=V + d + R)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=R)
    for head, alpha in ((0, 0.3), (1, 0.75)):
        kl = torch.full((R,), float("nan"), device=DEV)
        ce = torch.full((R,), float("nan"), device=DEV)
        loss = torch.full((3,), float("nan"), device=DEV)
        B.eh_head_losses(ctx, head, hid.h[head], hid.h[2], labels, R, alpha, kl, ce, loss)
        torch.cuda.synchronize()
        want = _oracle_losses(heads, hid, head, labels, alpha)
        kg, cg, lg = kl.double().cpu().numpy(), ce.double().cpu().numpy(), loss.double().cpu().numpy()
        assert _close(kg, want["kl"]).all(), (head, np.abs(kg - want["kl"]).max())
        assert _close(cg, want["ce"]).all(), (head, np.abs(cg - want["ce"]).max())
        assert _close(lg, np.array([want["L_ce"], want["L_kl"], want["L_hyb"]])).all(), (lg, want["L_ce"], want["L_kl"])
        assert (kg > -TOL_LOSS_ABS).all()
    B.eh_destroy(ctx)


def test_head_losses_special_cases(B):
    V, d, R = 600, 128, 70
    w, heads, hid, labels = _loss_case(V, d, R, seed=99)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=R)
    loss = torch.zeros(3, device=DEV)
    kl = torch.zeros(R, device=DEV)
    ce = torch.zeros(R, device=DEV)
    # the model's head against itself: no divergence; alpha = 1 leaves the cross-entropy alone
    B.eh_head_losses(ctx, 2, hid.h[2], hid.h[2], labels, R, 1.0, kl, ce, loss)
    torch.cuda.synchronize()
    want = _oracle_losses(heads, hid, 2, labels, 1.0)
    assert kl.abs().max().item() <= 1e-5 and abs(loss[1].item()) <= 1e-5
    assert _close(ce.double().cpu().numpy(), want["ce"]).all() and abs(loss[2].item() - loss[0].item()) <= 1e-6
    # no labels: the divergence is unchanged, every cross-entropy term is NaN, and so are L_CE and L_hyb
    B.eh_head_losses(ctx, 0, hid.h[0], hid.h[2], None, R, 0.5, kl, ce, loss)
    torch.cuda.synchronize()
    want = _oracle_losses(heads, hid, 0, None, 0.5)
    assert _close(kl.double().cpu().numpy(), want["kl"]).all() and torch.isnan(ce).all()
    assert math.isnan(loss[0].item()) and math.isnan(loss[2].item()) and _close(loss[1].item(), want["L_kl"])
    # per-token outputs are optional; a strided view of the hidden states is accepted
    wide = torch.zeros((R, 2 * d), dtype=hid.h.dtype, device=DEV)
    wide[:, :d] = hid.h[0]
    B.eh_head_losses(ctx, 0, wide[:, :d], hid.h[2], labels, R, 0.5, None, None, loss)
    torch.cuda.synchronize()
    want = _oracle_losses(heads, hid, 0, labels, 0.5)
    assert _close(loss.double().cpu().numpy(), np.array([want["L_ce"], want["L_kl"], want["L_hyb"]])).all()
    # a label outside the vocabulary gives that token a NaN cross-entropy, nothing else changes
    bad = labels.clone()
    bad[3] = V + 7
    bad[4] = -1
    B.eh_head_losses(ctx, 0, hid.h[0], hid.h[2], bad, R, 0.5, kl, ce, loss)
    torch.cuda.synchronize()
    c = ce.double().cpu().numpy()
    assert np.isnan(c[3]) and np.isnan(c[4]) and _close(np.delete(c, [3, 4]), np.delete(want["ce"], [3, 4])).all()
    assert _close(kl.double().cpu().numpy(), want["kl"]).all()
    with pytest.raises(B.EhError):
        B.eh_head_losses(ctx, 0, hid.h[0], hid.h[2], labels, 0, 0.5, None, None, loss)
    with pytest.raises(B.EhError):
        B.eh_head_losses(ctx, 5, hid.h[0], hid.h[2], labels, R, 0.5, None, None, loss)
    B.eh_destroy(ctx)


def test_head_losses_calibration_shape(B):
    """Config 2's shape (d = 2048, V = 50304, 512 tokens): two exit heads against the model's head;
    the oracle checks 40 sampled tokens per head, the means are checked for consistency with the
    library's own per-token terms (fp64 mean of the returned values)."""
    w = G.CONFIGS["c2_calib"]
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    R, fin = w.rows, w.n_heads - 1
    gen = torch.Generator(device=DEV)
    gen.manual_seed(4242)
    labels = torch.randint(0, w.V, (R,), generator=gen, device=DEV, dtype=torch.int32)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=R)
    sample = torch.arange(3, R, 13, device=DEV)[:40]
    f = P.f64
    Wt, gt, bt = f(heads.W[fin]), f(heads.gamma[fin]), f(heads.beta[fin])
    for head in (2, 17):
        kl = torch.zeros(R, device=DEV)
        ce = torch.zeros(R, device=DEV)
        loss = torch.zeros(3, device=DEV)
        B.eh_head_losses(ctx, head, hid.h[head], hid.h[fin], labels, R, 0.25, kl, ce, loss)
        torch.cuda.synchronize()
        want = O.head_losses(f(hid.h[head][sample]), f(hid.h[fin][sample]), f(heads.gamma[head]), f(heads.beta[head]),
                             f(heads.W[head]), gt, bt, Wt, labels[sample].cpu().numpy(), 0.25, 1e-5, True)
        kg, cg = kl[sample].double().cpu().numpy(), ce[sample].double().cpu().numpy()
        assert _close(kg, want["kl"]).all(), (head, np.abs(kg - want["kl"]).max())
        assert _close(cg, want["ce"]).all(), (head, np.abs(cg - want["ce"]).max())
        L_kl, L_ce = kl.double().mean().item(), ce.double().mean().item()
        assert abs(loss[1].item() - L_kl) <= 1e-5 * max(1.0, abs(L_kl))
        assert abs(loss[0].item() - L_ce) <= 1e-5 * max(1.0, abs(L_ce))
        assert abs(loss[2].item() - (0.25 * L_ce + 0.75 * L_kl)) <= 1e-5 * max(1.0, abs(L_ce))
        assert (kl > -TOL_LOSS_ABS).all() and torch.isfinite(kl).all() and torch.isfinite(ce).all()
        print(f"head {head}: L_CE {loss[0].item():.4f} L_KL {loss[1].item():.4f}")
    B.eh_destroy(ctx)


def test_dssd_draft_decode_shape(B):
    """The decode workload's heads (d = 1024, V = 50304, 24 heads), windows of 32 positions as
    bench.py drafts them: the oracle's cascade, position by position until the draft stops,
    feeds its drafting rule; a window in which an entropy the decision hinged on lies within
    1e-3 of its threshold is logged and skipped."""
    w = G.CONFIGS["c1_decode"]
    heads = G.make_heads(w, DEV)
    limit, n_win = 32, 6
    hid = G.make_hidden(w, heads, DEV, rows=limit * n_win)
    tau = G.tau_linear(w)
    f = P.f64
    W64 = [f(x) for x in heads.W]
    g64 = [f(x) for x in heads.gamma]
    b64 = [f(x) for x in heads.beta]
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, tau, max_rows=1)
    hp = hid.h.permute(1, 0, 2)
    checked, skipped = 0, []
    for i in range(n_win):
        draft = torch.full((limit,), -7, dtype=torch.int32, device=DEV)
        layers = torch.full((limit,), -7, dtype=torch.int32, device=DEV)
        ln = torch.zeros(1, dtype=torch.int32, device=DEV)
        reason = torch.zeros(1, dtype=torch.int32, device=DEV)
        fb = torch.zeros(1, dtype=torch.int32, device=DEV)
        nev = torch.zeros(1, dtype=torch.int64, device=DEV)
        B.dssd_draft(ctx, hp[i * limit:(i + 1) * limit], limit, -1, draft, ln, layers, reason, fb, nev)
        torch.cuda.synchronize()
        B.eh_check(ctx)
        Ht, At, close = [], [], False
        for t in range(i * limit, (i + 1) * limit):
            r = O.cascade([f(hid.h[l, t:t + 1]) for l in range(w.n_heads)], g64, b64, W64, tau, w.ln_eps, True)
            e = int(r["exit_layer"][0])
            Hrow = [float(r["H"][l][0]) if l <= e else float("nan") for l in range(w.n_heads)]
            close = close or any(abs(Hrow[l] - tau[l]) < 1e-3 for l in range(min(e + 1, w.n_heads - 1)))
            close = close or float(r["gap"][e][0]) < 1e-3
            Ht.append(Hrow)
            At.append([int(r["token"][0]) if l == e else -1 for l in range(w.n_heads)])
            if e == w.n_heads - 1:
                break
        if close:
            skipped.append(i)
            continue
        want = O.dssd_draft(Ht, At, tau, limit, -1)
        n = int(ln.item())
        got = dict(draft=draft[:n].tolist(), exit_layer=layers[:n].tolist(), reason=B.DRAFT_REASONS[int(reason.item())],
                   fallback_token=int(fb.item()), n_evals=int(nev.item()))
        assert got == want, (i, got, want)
        checked += 1
    print(f"draft windows checked {checked}, skipped for near-ties {skipped}")
    assert checked >= n_win - 2
    B.eh_destroy(ctx)


@pytest.mark.parametrize("kind", ["uniform", "few_values", "wide_range", "rounded", "signed_and_infinite", "narrow"])
def test_calibrate_random_sets_against_the_definition(B, small_ctx, kind):
    """Many small seeded sets of every shape the key range can take (a few distinct values, one
    binade, forty decades, negative and infinite 'entropies', which the interface does not
    forbid), each against the oracle's literal quadratic definition, bit for bit."""
    rng = np.random.default_rng({"uniform": 1, "few_values": 2, "wide_range": 3, "rounded": 4,
                                 "signed_and_infinite": 5, "narrow": 6}[kind])
    for trial in range(25):
        M = int(rng.integers(1, 500))
        if kind == "uniform":
            H = rng.uniform(0, 8, M)
        elif kind == "few_values":
            H = rng.choice(rng.uniform(0, 8, int(rng.integers(1, 7))), M)
        elif kind == "wide_range":
            H = np.abs(rng.normal(0, 1, M)) * 10.0 ** rng.integers(-20, 20, M)
        elif kind == "rounded":
            H = np.round(rng.uniform(0, 4, M), 1)
        elif kind == "signed_and_infinite":
            H = rng.normal(0, 3, M)
            H[rng.random(M) < 0.05] = np.inf
            H[rng.random(M) < 0.05] = -np.inf
            H[rng.random(M) < 0.05] = 0.0
            H[rng.random(M) < 0.05] = -0.0
        else:
            H = 3.0 + rng.integers(0, 300, M) * 2.0 ** -21         # a few hundred neighbouring floats
        H = H.astype(np.float32)
        if trial % 5 == 0:
            H[rng.integers(0, M)] = np.nan
        finite = np.where(np.isfinite(H), H, 0.0)
        p = rng.uniform(0.2, 0.95)
        ok = rng.random(M) < np.clip(p + 0.3 * (finite < np.median(finite)), 0, 1)
        ref = np.ones(M, np.int32)
        pred = np.where(ok, 1, 2).astype(np.int32)
        eps = [0.0, 0.5, 0.7, 0.9, 1.0, float(rng.uniform(0, 1)), float(rng.uniform(0, 1))]
        tau, n = _calibrate(B, small_ctx, torch.tensor(H, device=DEV), torch.tensor(pred, device=DEV),
                            torch.tensor(ref, device=DEV), eps)
        Hc = H.astype(np.float64)
        for i, e in enumerate(eps):
            want_tau, want_n = O.calibrate_threshold(Hc, ok, e)
            same = (tau[i] == np.float32(want_tau)) or (np.isneginf(tau[i]) and np.isneginf(want_tau))
            assert same and int(n[i]) == want_n, (kind, trial, M, e, tau[i], want_tau, n[i], want_n)


def test_calibrate_data_that_cannot_be_pruned_is_sorted(B, small_ctx):
    """Distinct entropies with predictions alternately wrong and right in order of entropy: the
    proportion among the c most confident tokens is 1/2 for even c and just under it for odd c.
    At a level a hair above 1/2 no threshold qualifies, but no bin of any level can be ruled
    out from its counts either (its bound lies above the level), so the tables of kept bins
    overflow and the call must notice and sort; at 1/2 itself the very top qualifies and the
    counting answers at once.  Both answers are checked, and which way each call went."""
    M = 1 << 16
    H = (torch.arange(M, device=DEV, dtype=torch.float32) * 1e-4 + 0.25)[torch.randperm(
        M, generator=torch.Generator(device="cpu").manual_seed(5)).to(DEV)].contiguous()
    rank = torch.argsort(torch.argsort(H))                              # position in ascending entropy
    ref = torch.zeros(M, dtype=torch.int32, device=DEV)
    pred = (1 - (rank % 2)).to(torch.int32)                             # even rank: wrong (1 != 0), odd: right
    Hc = H.cpu().numpy().astype(np.float64)
    t = O.correctness(pred.cpu().numpy(), ref.cpu().numpy())
    for eps, sorts in (([0.5], 0), ([0.5000001], 1), ([0.5, 0.5000001, 0.3], 1)):
        before = B.eh_probe_calibrate_sorted(small_ctx)
        tau, n = _calibrate(B, small_ctx, H, pred, ref, eps)
        assert B.eh_probe_calibrate_sorted(small_ctx) - before == sorts, eps
        for i, (want_tau, want_n) in enumerate(_calibrate_by_counting(Hc, t, eps)):
            assert tau[i] == want_tau and n[i] == want_n, (eps[i], tau[i], want_tau, n[i], want_n)
    assert np.isneginf(_calibrate(B, small_ctx, H, pred, ref, [0.5000001])[0][0])
