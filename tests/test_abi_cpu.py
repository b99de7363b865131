"""Host-side checks that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching a device."""
import ctypes as C
import math
import os
import re

import pytest

from paper_2407_21082_amd import binding as B
from workloads import generators as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header="eh.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(eh_[a-z0-9_]+|dssd_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    probes = _declared("eh_probe.h")
    assert set(probes) == set(B.PROBE_EXPORTS)
    for n in names + probes:
        assert hasattr(B.lib, n), f"libeh.so does not export {n}"
    assert "gfx950" in B.eh_version()
    # nothing else with the library's prefixes is exported (diagnostic hooks stay out of the default build)
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", B.LIB_PATH], stdout=subprocess.PIPE, text=True, check=True).stdout
    exported = {l.split()[-1] for l in out.splitlines() if " T " in l}
    ours = {n for n in exported if n.startswith(("eh_", "dssd_"))}
    assert ours == set(names) | set(probes), ours ^ (set(names) | set(probes))


def _cfg(**kw):
    one = (C.c_void_p * 1)(16)
    tau = (C.c_float * 1)(1.0)
    base = dict(d=64, V=100, n_heads=1, max_rows=4, w_dtype=B.EH_BF16, h_dtype=B.EH_BF16, ln_eps=1e-5,
                device=0, W=one, gamma=one, beta=one, bias=None, tau=tau)
    base.update(kw)
    return B._Config(**base)


@pytest.mark.parametrize("kw,status", [
    (dict(d=0), 2), (dict(V=-1), 2), (dict(n_heads=0), 2), (dict(max_rows=0), 2),
    (dict(w_dtype=7, h_dtype=7), 3), (dict(h_dtype=B.EH_F32), 3), (dict(d=12), 2),
    (dict(ln_eps=0.0), 4), (dict(W=None), 1), (dict(tau=None), 1),
    (dict(W=(C.c_void_p * 1)(8)), 2),          # misaligned weight pointer
])
def test_create_rejects_bad_config_on_host(kw, status):
    out = C.c_void_p()
    st = B.lib.eh_create(C.byref(_cfg(**kw)), C.byref(out))
    assert st == status and not out.value
    assert B.lib.eh_last_error(None)           # a message is always available


def test_null_arguments():
    assert B.lib.eh_create(None, None) == 1
    assert B.lib.eh_destroy(None) == 1
    assert B.lib.eh_eval(None, 0, None, 0, None, None, 0, None, None, None, None) == 1
    assert B.lib.dssd_verify(None, None, None, None, 1, 1, None, None, None, None) == 1
    assert B.lib.eh_eval_heads(None, 0, 1, None, 0, 0, 1, None, None, None, None) == 1
    assert B.lib.eh_eval_heads_metrics(None, 0, 1, None, 0, 0, 1, None, None, None, None, None, None) == 1
    assert B.lib.eh_cascade(None, None, 0, 0, 1, None, None, None, None, None) == 1
    assert B.lib.dssd_draft(None, None, 0, 0, 1, 1, -1, None, None, None, None, None, None, None) == 1
    assert B.lib.dssd_tally(None, None, None, 1, 1, None, None, None) == 1
    assert B.lib.eh_head_losses(None, 0, None, 0, None, 0, None, 1, 0.5, None, None, None, None) == 1
    assert B.lib.eh_calibrate(None, None, None, None, 1, None, 1, None, None, None) == 1


# ---------------------------------------------------------------- repository rules, checked on the tree
def _sources(*dirs, exts=(".py", ".hip", ".hpp", ".h")):
    for d in dirs:
        for base, _, files in os.walk(os.path.join(ROOT, d)):
            if "_build" in base or "__pycache__" in base:
                continue
            for f in files:
                if f.endswith(exts):
                    yield os.path.join(base, f)


WORK = "_" + "work/"      # spelled so that this file does not name the folder itself


def test_product_never_touches_the_oracle_or_working_files():
    """The library and its binding are the product: no import of the oracle, no CPU fallback module,
    nothing read from the working folder."""
    for path in _sources("paper_2407_21082_amd", "include"):
        text = open(path).read()
        assert "oracle" not in text.lower() or path.endswith("check_gemm_asm.py"), path
        assert WORK not in text, path
    for path in list(_sources("tests", "oracle", "workloads")) + [os.path.join(ROOT, "bench.py"),
                                                                   os.path.join(ROOT, "__graft_entry__.py")]:
        assert WORK not in open(path).read(), path
    # the oracle in turn imports nothing of the product
    for path in _sources("oracle"):
        assert "paper_2407_21082_amd" not in open(path).read(), path


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0 and "single-GPU" in r.stderr and r.stdout.strip() == ""


# ---------------------------------------------------------------- generators
def test_generators_are_seeded_and_shaped():
    w = G.Workload("t", d=64, V=500, n_heads=3, rows=10, dtype="bf16", seed=3)
    a, b = G.make_heads(w), G.make_heads(w)
    assert all((x == y).all() for x, y in zip(a.W, b.W))
    assert a.W[0].shape == (500, 64) and a.gamma[0].dtype.is_floating_point
    h1, h2 = G.make_hidden(w, a), G.make_hidden(w, b)
    assert (h1.h == h2.h).all() and h1.h.shape == (3, 10, 64)
    assert (h1.s >= w.s_lo).all() and (h1.s <= w.s_hi).all()
    tau = G.tau_linear(w)
    assert tau[0] == pytest.approx(0.5) and tau[1] == pytest.approx(3.0) and math.isinf(tau[2])


def test_tau_for_schedule_follows_the_fractions():
    import numpy as np
    rng = np.random.default_rng(0)
    n, R = 32, 64
    H = np.sort(rng.uniform(0, 10, size=(n, R)), axis=0)[::-1] + rng.uniform(0, 1e-3, size=(n, R))
    tau = G.tau_for_schedule(H, n)
    active = np.ones(R, bool)
    for l in range(n - 1):
        active &= ~(H[l] < tau[l])
        want = round(G.exit_schedule_fraction(l, n) * R)
        assert abs((R - active.sum()) - want) <= 1
    assert G.exit_schedule_fraction(7, 32) == pytest.approx(0.10)
    assert G.exit_schedule_fraction(15, 32) == pytest.approx(0.40)
    assert G.exit_schedule_fraction(23, 32) == pytest.approx(0.70)
