"""The entry point that allocates nothing (eh_eval_noalloc: eh_eval on the library's static
workspace) against eh_eval itself, through the C ABI: two calls in a row, the second with a
smaller input, so that the second meets the first one's leftovers in the shared array."""
import numpy as np
import pytest
import torch

from workloads import generators as G
from tests import parity_util as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _outs(n):
    return (torch.full((n,), float("nan"), device=DEV), torch.full((n,), float("nan"), device=DEV),
            torch.full((n,), -7, dtype=torch.int32, device=DEV))


def _same(name, a, b, bitwise):
    """eh_eval's outputs `a` against the variant's `b`: index exact; entropy and log-sum-exp
    to the parity tolerances (bit for bit where both calls run the same kernels)."""
    Ha, La, Aa = a
    Hb, Lb, Ab = b
    assert torch.equal(Aa, Ab), name
    if bitwise:
        assert torch.equal(Ha.view(torch.int32), Hb.view(torch.int32)) and torch.equal(La.view(torch.int32), Lb.view(torch.int32)), name
    dH = (Ha.double() - Hb.double()).abs().max().item()
    dl = ((La.double() - Lb.double()).abs() / La.double().abs().clamp_min(1.0)).max().item()
    assert dH <= P.TOL_H and dl <= P.TOL_LSE_REL, (name, dH, dl)


@pytest.mark.parametrize("dtype,d,V,first,second", [("bf16", 256, 3000, 70, 33), ("bf16", 2560, 50304, 150, 64),
                                                    ("f32", 128, 2000, 40, 20), ("bf16", 256, 3000, 40, 9)])
def test_noalloc_matches_eh_eval_on_two_calls_in_a_row(dtype, d, V, first, second):
    from paper_2407_21082_amd import binding as B
    w = G.Workload("noalloc", d=d, V=V, n_heads=2, rows=first, dtype=dtype, seed=first + second)
    heads = G.make_heads(w, DEV)
    hid = G.make_hidden(w, heads, DEV)
    ctx = B.eh_create(heads.W, heads.gamma, heads.beta, G.tau_linear(w), max_rows=first)
    for head, rows in ((0, first), (1, second)):
        want = _outs(rows)
        B.eh_eval(ctx, head, hid.h[head], rows, *want)
        got = _outs(rows)
        B.eh_eval_noalloc(ctx, head, hid.h[head], rows, *got)
        torch.cuda.synchronize()
        B.eh_check(ctx)
        assert torch.isfinite(got[0]).all() and (got[2] >= 0).all()
        # more than 16 rows: eh_eval runs the same kernels; at most 16 it runs the persistent one
        _same(f"{dtype}/{rows}", want, got, bitwise=rows > 16)
    # a gather list and a device-side row count, as eh_eval takes them
    idx = torch.arange(second - 1, -1, -1, dtype=torch.int32, device=DEV)
    n_dev = torch.tensor([second - 3], dtype=torch.int32, device=DEV)
    want, got = _outs(second), _outs(second)
    B.eh_eval(ctx, 0, hid.h[0], second, *want, row_idx=idx, n_rows_dev=n_dev)
    B.eh_eval_noalloc(ctx, 0, hid.h[0], second, *got, row_idx=idx, n_rows_dev=n_dev)
    torch.cuda.synchronize()
    live = second - 3
    _same("gather", tuple(x[:live] for x in want), tuple(x[:live] for x in got), bitwise=second > 16)
    assert torch.isnan(got[0][live:]).all() and (got[2][live:] == -7).all()      # dead positions untouched
    # sizes beyond the static array are refused before anything is launched; nothing else changes
    huge = torch.zeros((1, d), dtype=hid.h.dtype, device=DEV)
    with pytest.raises(B.EhError) as e:
        B.eh_eval_noalloc(ctx, 0, huge, 1 << 19, None, None, None)
    assert e.value.status == 6
    B.eh_eval_noalloc(ctx, 0, huge, 0, None, None, None)                           # no rows: a no-op
    B.eh_destroy(ctx)
