"""Seeded synthetic workloads with the shapes of the Pythia family.

The paper (arXiv 2407.21082, Section 4) evaluates on Pythia checkpoints, heads
trained on MiniPile and public benchmarks; none of that is available here, so
these generators stand in for it: they take only the shapes (hidden size d,
padded vocabulary 50304, number of layers) and produce random heads and hidden
states whose head outputs span the whole range of entropies, so that the
calibrated exit rule (Section 3.4.2) fires at many different depths.

Recipe (per head l, per token t):

    W_l[i, :] ~ N(0, 1/d)           gamma = 1 + 0.02 N(0,1)    beta = 0.02 N(0,1)
    g ~ N(0, 1)^d                   c_t ~ Uniform{0..V-1}      s_t ~ LogUniform(s_lo, s_hi)
    w^ = W_l[c_t] / ||W_l[c_t]||    a = kappa * s_t * rho(l)   rho(l) = (l + 1) / n_heads
    h[l, t, :] = s_t * (g + a * sqrt(d) * w^)

The per-token scale s_t alone would be erased by LayerNorm; tying the strength
of a planted direction (the token's "true" next token c_t) to s_t and to depth
is what spreads the entropies: after LayerNorm the planted logit is about
sqrt(d) * a / sqrt(1 + a^2) over a unit-variance background.

Nothing here computes any step of the method; the module only draws numbers.
All tensors are torch tensors on the requested device, drawn from a seeded
``torch.Generator`` of that device, so a run is reproducible on a given device
type.  Consumers hand the very same stored values to both the oracle and the
HIP path.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional

import torch

V_PYTHIA = 50304


@dataclass(frozen=True)
class Workload:
    name: str
    d: int
    V: int
    n_heads: int            # exit heads + the final head (last)
    rows: int               # tokens per head evaluation
    dtype: str              # "bf16" or "f32" (storage of W and h)
    s_lo: float = 0.5
    s_hi: float = 8.0
    kappa: float = 0.25
    tau_lo: float = 0.5
    tau_hi: float = 3.0
    steps: int = 1          # independent decode steps (config 1)
    seed: int = 20240721
    ln_eps: float = 1e-5

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


# The five configurations of the build, plus reduced shapes for quick checks.
CONFIGS = {
    "c0_tiny": Workload("c0_tiny", d=512, V=V_PYTHIA, n_heads=6, rows=32, dtype="f32"),
    "c1_decode": Workload("c1_decode", d=1024, V=V_PYTHIA, n_heads=24, rows=1, dtype="bf16", steps=2048),
    "c2_calib": Workload("c2_calib", d=2048, V=V_PYTHIA, n_heads=24, rows=512, dtype="bf16",
                         s_lo=0.25, s_hi=16.0),
    "c3_dynexit": Workload("c3_dynexit", d=2560, V=V_PYTHIA, n_heads=32, rows=64, dtype="bf16"),
    "c4_verify": Workload("c4_verify", d=2560, V=V_PYTHIA, n_heads=32, rows=16 * 9, dtype="bf16"),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (reduced shapes for tests)."""
    return replace(w, **kw)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, gen, device, chunk_rows: int = 8192):
    """N(0,1) fp32 tensor drawn in row chunks (bounds transient memory)."""
    out = torch.empty(shape, dtype=torch.float32, device=device)
    flat = out.view(shape[0], -1) if len(shape) > 1 else out.view(-1, 1)
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        flat[r0:r1] = torch.randn((r1 - r0, flat.shape[1]), generator=gen, device=device,
                                  dtype=torch.float32)
    return out


@dataclass
class Heads:
    W: List[torch.Tensor]        # n_heads x [V, d] in the workload dtype
    gamma: List[torch.Tensor]    # n_heads x [d] fp32
    beta: List[torch.Tensor]     # n_heads x [d] fp32


def make_heads(w: Workload, device="cpu", n_heads: Optional[int] = None) -> Heads:
    n = w.n_heads if n_heads is None else n_heads
    Ws, gs, bs = [], [], []
    for l in range(n):
        gen = _gen(device, w.seed * 1000 + l)
        Wl = _randn((w.V, w.d), gen, device) * (1.0 / math.sqrt(w.d))
        Ws.append(Wl.to(w.torch_dtype).contiguous())
        gs.append((1.0 + 0.02 * torch.randn(w.d, generator=gen, device=device)).float().contiguous())
        bs.append((0.02 * torch.randn(w.d, generator=gen, device=device)).float().contiguous())
    return Heads(Ws, gs, bs)


def rho(l: int, n_heads: int) -> float:
    return (l + 1) / n_heads


@dataclass
class Hidden:
    h: torch.Tensor          # [n_heads, rows, d] in the workload dtype
    planted: torch.Tensor    # [rows] int64, the token each row is aligned with
    s: torch.Tensor          # [rows] fp32 per-token scale


def make_hidden(w: Workload, heads: Heads, device="cpu", rows: Optional[int] = None,
                seed_offset: int = 0, planted: Optional[torch.Tensor] = None,
                amp: Optional[torch.Tensor] = None, layers: Optional[List[int]] = None) -> Hidden:
    """Hidden states for every head of ``heads`` (or for ``layers`` only).

    ``planted`` overrides the per-row planted token; ``amp`` overrides the
    planted amplitude a (per row, the same at every layer) -- used by the
    verification workload, whose final hidden states must decide clearly.
    """
    R = w.rows if rows is None else rows
    gen = _gen(device, w.seed * 7 + 1 + seed_offset)
    u = torch.rand(R, generator=gen, device=device)
    s = torch.exp(math.log(w.s_lo) + u * (math.log(w.s_hi) - math.log(w.s_lo)))
    if planted is None:
        planted = torch.randint(0, w.V, (R,), generator=gen, device=device)
    else:
        torch.randint(0, w.V, (R,), generator=gen, device=device)  # keep the stream aligned
        planted = planted.to(device)
    ls = list(range(len(heads.W))) if layers is None else layers
    n_total = len(heads.W)
    out = torch.empty((len(ls), R, w.d), dtype=w.torch_dtype, device=device)
    for i, l in enumerate(ls):
        g = torch.randn((R, w.d), generator=gen, device=device)
        rows_w = heads.W[l][planted].float()
        w_hat = rows_w / rows_w.norm(dim=1, keepdim=True)
        a = (w.kappa * s * rho(l, n_total)) if amp is None else amp.to(device)
        hl = s[:, None] * (g + (a * math.sqrt(w.d))[:, None] * w_hat)
        out[i] = hl.to(w.torch_dtype)
    return Hidden(out, planted, s)


def tau_linear(w: Workload, n_heads: Optional[int] = None) -> List[float]:
    """Thresholds rising linearly over the exit heads; the last head (the full
    model) ignores its entry."""
    n = w.n_heads if n_heads is None else n_heads
    k = n - 1
    if k <= 0:
        return [float("inf")]
    taus = [w.tau_lo + (w.tau_hi - w.tau_lo) * (i / max(1, k - 1)) for i in range(k)]
    return taus + [float("inf")]


def exit_schedule_fraction(head: int, n_heads: int) -> float:
    """Target cumulative fraction of rows that have exited after ``head``:
    piecewise linear through 0 % at the start, 10 / 40 / 70 % after a quarter,
    half and three quarters of the depth, and 90 % before the final head."""
    x = (head + 1) / n_heads
    pts = [(0.0, 0.0), (0.25, 0.10), (0.50, 0.40), (0.75, 0.70), (1.0, 0.90)]
    for (x0, y0), (x1, y1) in zip(pts[:-1], pts[1:]):
        if x <= x1:
            return y0 + (y1 - y0) * (x - x0) / (x1 - x0)
    return pts[-1][1]


def tau_for_schedule(H, n_heads: int) -> List[float]:
    """Thresholds that make a given table of entropies H[l][r] (a plain nested
    sequence or array: every head on every row) follow ``exit_schedule_fraction``.

    Walks the heads shallow to deep keeping the set of rows still active; at
    head l it puts tau_l midway between the n-th and (n+1)-th smallest entropy
    among active rows, n being the number of exits still owed to the schedule,
    so that every |H - tau| margin is as wide as the data allows.  Pure order
    statistics on numbers handed in; where they come from is the caller's
    business (the tests hand in the CPU oracle's entropies).
    """
    R = len(H[0])
    active = list(range(R))
    exited = 0
    taus: List[float] = []
    for l in range(n_heads - 1):
        want = int(round(exit_schedule_fraction(l, n_heads) * R)) - exited
        vals = sorted((float(H[l][r]), r) for r in active)
        n = max(0, min(want, len(vals)))
        if not vals:
            taus.append(0.0)
            continue
        if n == 0:
            t = vals[0][0] - 0.5
        elif n == len(vals):
            t = vals[-1][0] + 0.5
        else:
            t = 0.5 * (vals[n - 1][0] + vals[n][0])
        taus.append(t)
        gone = {r for v, r in vals if v < t}
        active = [r for r in active if r not in gone]
        exited += len(gone)
    return taus + [float("inf")]


@dataclass
class VerifyCase:
    f_final: torch.Tensor    # [B, k+1, d]
    agree: torch.Tensor      # [B, k+1] bool: position planted with the draft token
    planted: torch.Tensor    # [B, k+1] int64 planted (intended) full-model token


def make_verify_case(w: Workload, heads: Heads, draft: torch.Tensor, device="cpu",
                     p_agree: float = 0.7, amp: float = 1.5, seed_offset: int = 991) -> VerifyCase:
    """Final-layer hidden states for DSSD verification (Section 4.3.1).

    draft is [B, k].  Position j < k is planted with draft[b, j] with
    probability ``p_agree`` and with an independent uniform token otherwise;
    position k (the bonus position) gets a uniform token.  The planted
    amplitude is large so the final head decides with a wide margin.
    """
    B, k = draft.shape
    gen = _gen(device, w.seed * 13 + seed_offset)
    agree = torch.rand((B, k + 1), generator=gen, device=device) < p_agree
    agree[:, k] = False
    other = torch.randint(0, w.V, (B, k + 1), generator=gen, device=device)
    planted = other.clone()
    planted[:, :k] = torch.where(agree[:, :k], draft.to(device).long(), other[:, :k])
    final = len(heads.W) - 1
    hid = make_hidden(w, heads, device, rows=B * (k + 1), seed_offset=seed_offset,
                      planted=planted.reshape(-1),
                      amp=torch.full((B * (k + 1),), amp, device=device), layers=[final])
    return VerifyCase(hid.h[0].reshape(B, k + 1, w.d).contiguous(), agree, planted)


def make_calibration_case(M: int, device="cpu", seed: int = 0, V: int = V_PYTHIA, ties: bool = False,
                          nan_every: int = 0):
    """Synthetic calibration set of one head (Section 3.4.1): entropies H[M] (float32, spread
    like a head's over text: a gamma-shaped bulk below ln V), the head's and the model's
    predictions pred[M], ref[M] (int32), with agreement the likelier the lower the entropy.
    ties=True quantises the entropies so that many tokens share a value; nan_every > 0 plants a
    NaN entropy at every nan_every-th token."""
    gen = _gen(device, 7919 * seed + 17)
    u = torch.rand((3, M), generator=gen, device=device)
    H = (-(torch.log(u[0].clamp_min(1e-12)) + torch.log(u[1].clamp_min(1e-12))) * 0.9).clamp(max=math.log(V))
    if ties:
        H = torch.round(H * 8) / 8
    H = H.to(torch.float32)
    p_agree = torch.exp(-0.9 * H)
    ref = torch.randint(0, V, (M,), generator=gen, device=device, dtype=torch.int64)
    other = (ref + 1 + torch.randint(0, V - 1, (M,), generator=gen, device=device, dtype=torch.int64)) % V
    pred = torch.where(u[2] < p_agree, ref, other)
    if nan_every > 0:
        H[::nan_every] = float("nan")
    return H.contiguous(), pred.to(torch.int32).contiguous(), ref.to(torch.int32).contiguous()


# ---------------------------------------------------------------- conversions
def to_f64_numpy(t: torch.Tensor):
    """The exact stored values of a tensor as a float64 numpy array (host)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
