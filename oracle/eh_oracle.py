"""CPU fp64 oracle for early-exit head evaluation and DSSD greedy verification.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP path is checked against.  It must never be imported by the product package;
only tests, the smoke check and the benchmark's cpu_baseline leg call it.  It
shares no code with the HIP path and imports nothing from it.

Everything is computed in numpy float64, two-pass, with the logits of a head
materialised in full -- the exact opposite of the streamed, fused, low-precision
formulation the kernels use.

What each function follows (arXiv 2407.21082):

* ``head_logits`` / ``layernorm``: Section 3.2, "Implementation Details": an
  exit head has the structure of the model's final classification head and is
  fed the hidden features of a transformer block.  For the Pythia family that
  is a LayerNorm followed by a bias-free d -> |V| linear map.
* ``softmax_stats``: Section 3.4.1: the confidence metric is the entropy of the
  predicted distribution, H(p) = -sum_j p_j log p_j (natural log, 0 log 0 = 0);
  eq. (2) uses argmax p, taken here with the lowest index on ties.
* ``exit_rule``: Section 3.4.2 (exit at the first head whose confidence passes
  its threshold, otherwise the full model's output) in the entropy form of
  Section 4.3.1, "Drafting phase": first head with H(p_k) < tau_k.
* ``dssd_verify``: Section 4.3.1, "Verification phase": every drafted token is
  compared with the full model's greedy prediction for its position; the
  accepted prefix is committed and the first mismatch is replaced by the
  full-model token.

* ``dssd_draft``: Section 4.3.1, "Drafting phase": position by position the first
  exit head whose entropy is under its threshold supplies the token, which is
  appended to the draft buffer, until the buffer is full, an end-of-sequence
  token has been drafted, or no exit head is confident (fallback to the model).
* ``dssd_tally``: Section 4.3.1, "Verification phase", and the figures of Section
  4.3.2: tokens drafted, committed and discarded over verification rounds, the
  acceptance rate (committed / drafted) and the mean accepted tokens per round.
* ``token_losses`` / ``head_losses``: Section 3.3, "Losses": the cross-entropy of the
  head's distribution against the labels, the Kullback-Leibler divergence of the
  head's distribution from the main model's (head first), their means over the
  sequence and the hybrid objective alpha L_CE + (1 - alpha) L_KL.  Forward only.
* ``confidence_metrics``: Section 3.4.1: the two confidence metrics the paper
  compares entropy with, the maximum probability and the difference between the
  two largest probabilities ("breaking ties").
* ``calibrate_threshold``: Section 3.4.1, "Calibration of Confidence Thresholds":
  correctness t_j from eq. (2), the joint sort by confidence, the smallest index
  whose suffix holds a proportion of correct predictions of at least epsilon,
  and tau = the confidence value at that index, with entropy as the metric.

Readings taken where the paper is silent (LayerNorm epsilon, biased variance,
where bf16 rounding happens, strict inequality, alignment of draft and target
positions) are listed in the repository's design notes; the ones that matter
here are repeated in the docstrings.

Parity pins: every function in this file is pinned by the CPU tests (closed
forms, invariants, exhaustive enumeration on tiny cases).  No function is
"parity unpinned".
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "bf16_bits_to_f64",
    "round_to_bf16",
    "f64_to_bf16_bits",
    "layernorm",
    "head_logits",
    "softmax_stats",
    "head_eval",
    "exit_rule",
    "cascade",
    "dssd_verify",
    "accepted_prefix",
    "dssd_draft",
    "dssd_tally",
    "confidence_metrics",
    "head_metrics",
    "correctness",
    "calibrate_threshold",
    "token_losses",
    "head_losses",
]


# ----------------------------------------------------------------------------
# bf16 <-> fp64 (storage format only; bf16 = sign, 8 exponent bits, 7 mantissa
# bits, i.e. the upper half of an IEEE binary32)
# ----------------------------------------------------------------------------
def bf16_bits_to_f64(bits) -> np.ndarray:
    """Exact value of bf16 bit patterns (uint16 array) as float64."""
    b = np.asarray(bits, dtype=np.uint16)
    as32 = (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
    with np.errstate(invalid="ignore"):      # signalling-NaN patterns
        return as32.astype(np.float64)


def round_to_bf16(x) -> np.ndarray:
    """Round float64 values to the nearest bf16-representable value, ties to
    even, returned as float64.

    Written from the definition of the format, not by bit tricks: a finite
    non-zero x with binary exponent e = floor(log2|x|) lies on a grid of
    spacing 2**(max(e, -126) - 7) (8 significant bits; below 2**-126 the grid
    is the subnormal one).  x / spacing is exact in fp64 (power-of-two scale),
    ``np.rint`` rounds half to even, and multiplying back is exact.  Results of
    magnitude >= 2**128 overflow to infinity.  NaN and +-inf pass through.
    """
    x = np.asarray(x, dtype=np.float64)
    out = x.copy()
    fin = np.isfinite(x) & (x != 0.0)
    if np.any(fin):
        xf = x[fin]
        _, ex = np.frexp(xf)              # xf = m * 2**ex with 0.5 <= |m| < 1
        e = ex.astype(np.int64) - 1        # floor(log2|xf|)
        q = np.ldexp(1.0, (np.maximum(e, -126) - 7).astype(np.int64))
        r = np.rint(xf / q) * q
        r = np.where(np.abs(r) >= np.ldexp(1.0, 128), np.copysign(np.inf, xf), r)
        out[fin] = r
    return out


def f64_to_bf16_bits(x) -> np.ndarray:
    """bf16 bit patterns (uint16) of values already representable in bf16."""
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = x32.view(np.uint32)
    if np.any((u & np.uint32(0xFFFF)) != 0):
        raise ValueError("value is not bf16-representable")
    return (u >> np.uint32(16)).astype(np.uint16)


# ----------------------------------------------------------------------------
# One head
# ----------------------------------------------------------------------------
def layernorm(h, gamma, beta, eps=1e-5, bf16_out=False) -> np.ndarray:
    """LayerNorm over the last axis in fp64, two-pass, biased variance:
    mu = mean(h); var = mean((h - mu)^2); y = gamma*(h - mu)/sqrt(var+eps)+beta.

    ``bf16_out`` rounds y to bf16 (ties to even): in bf16 mode the normalised
    activations are the low-precision operand of the projection, and both
    sides of the parity check agree that this is where the rounding happens.
    """
    h = np.asarray(h, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    d = h.shape[-1]
    mu = h.sum(axis=-1, keepdims=True) / d
    c = h - mu
    var = (c * c).sum(axis=-1, keepdims=True) / d
    y = gamma * (c / np.sqrt(var + eps)) + beta
    if bf16_out:
        y = round_to_bf16(y)
    return y


def head_logits(y, W, bias=None) -> np.ndarray:
    """z[r, i] = sum_j W[i, j] * y[r, j] (+ bias[i]); W is [V, d]."""
    y = np.asarray(y, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    z = y @ W.T
    if bias is not None:
        z = z + np.asarray(bias, dtype=np.float64)
    return z


def softmax_stats(z):
    """Entropy, log-sum-exp, argmax and top-2 gap of each row of logits.

    Two passes over materialised logits, straight from the definitions:
    m = max z; S = sum exp(z - m); lse = m + log S; p = exp(z - lse);
    H = -sum_{p>0} p * log p with log p = z - lse; argmax = lowest index
    attaining m; gap = m - (second largest logit, counting multiplicity).
    Returns (H, lse, argmax, gap); a NaN anywhere in a row gives NaN H/lse.
    """
    z = np.asarray(z, dtype=np.float64)
    if z.ndim == 1:
        z = z[None, :]
    R, V = z.shape
    H = np.empty(R)
    lse = np.empty(R)
    am = np.empty(R, dtype=np.int64)
    gap = np.empty(R)
    for r in range(R):
        zr = z[r]
        m = zr.max()
        if not np.isfinite(m):
            H[r] = lse[r] = gap[r] = np.nan
            am[r] = -1
            continue
        S = np.exp(zr - m).sum()
        L = m + np.log(S)
        logp = zr - L
        p = np.exp(logp)
        keep = p > 0.0
        H[r] = -(p[keep] * logp[keep]).sum()
        lse[r] = L
        am[r] = np.flatnonzero(zr == m)[0]
        if V > 1:
            rest = np.delete(zr, am[r])
            gap[r] = m - rest.max()
        else:
            gap[r] = np.inf
    return H, lse, am, gap


def confidence_metrics(z):
    """Maximum probability and top-2 probability difference of each row of logits
    (Section 3.4.1, metrics (1) and (3)).

    Straight from the definitions on the materialised distribution: p = softmax(z)
    computed as exp(z - lse); the probabilities are sorted, max_prob is the largest
    and margin the largest minus the second largest (a tie at the top gives 0; with
    a single class the second largest probability is taken as 0).  A row with a NaN
    or without a finite maximum gives NaN.  Returns (max_prob, margin).
    """
    z = np.asarray(z, dtype=np.float64)
    if z.ndim == 1:
        z = z[None, :]
    R, V = z.shape
    pmax = np.empty(R)
    margin = np.empty(R)
    for r in range(R):
        zr = z[r]
        m = zr.max()
        if not np.isfinite(m):
            pmax[r] = margin[r] = np.nan
            continue
        L = m + np.log(np.exp(zr - m).sum())
        p = np.sort(np.exp(zr - L))
        pmax[r] = p[-1]
        margin[r] = p[-1] - (p[-2] if V > 1 else 0.0)
    return pmax, margin


def head_metrics(h, gamma, beta, W, eps=1e-5, bf16=False, bias=None):
    """LayerNorm -> projection -> (max_prob, margin) for rows h [R, d]."""
    y = layernorm(h, gamma, beta, eps, bf16_out=bf16)
    return confidence_metrics(head_logits(y, W, bias))


def head_eval(h, gamma, beta, W, eps=1e-5, bf16=False, bias=None):
    """LayerNorm -> projection -> softmax statistics for rows h [R, d].

    Inputs are the very values the device receives, already widened to fp64
    (bf16 inputs via ``bf16_bits_to_f64``).  Returns (H, lse, argmax, gap).
    """
    y = layernorm(h, gamma, beta, eps, bf16_out=bf16)
    z = head_logits(y, W, bias)
    return softmax_stats(z)


# ----------------------------------------------------------------------------
# Exit rule and cascade
# ----------------------------------------------------------------------------
def exit_rule(H_by_head, tau) -> int:
    """Index of the head a token exits at: the first k < n_heads-1 with
    H_k < tau_k (strict), else the last head, which stands for the full model
    and always answers.  NaN entropies never pass the test."""
    n = len(H_by_head)
    for k in range(n - 1):
        if H_by_head[k] < tau[k]:
            return k
    return n - 1


def cascade(h_layers, gammas, betas, Ws, tau, eps=1e-5, bf16=False):
    """Dynamic-exit inference for R independent rows.

    h_layers[l] is [R, d], the hidden state each head sees.  Heads are visited
    shallow to deep; head l is evaluated only on the rows that have not yet
    exited (the increasing list of their indices is the active list after
    compaction).  Returns dict with exit_layer[R], token[R], H[n_heads, R],
    lse, argmax, gap (NaN / -1 where a row was no longer active) and
    active[l] = the index list head l was evaluated on.
    """
    n_heads = len(Ws)
    R = np.asarray(h_layers[0]).shape[0]
    H = np.full((n_heads, R), np.nan)
    lse = np.full((n_heads, R), np.nan)
    am = np.full((n_heads, R), -1, dtype=np.int64)
    gap = np.full((n_heads, R), np.nan)
    exit_layer = np.full(R, -1, dtype=np.int64)
    token = np.full(R, -1, dtype=np.int64)
    active = np.arange(R)
    actives = []
    for l in range(n_heads):
        actives.append(active.copy())
        if active.size == 0:
            continue
        hl = np.asarray(h_layers[l], dtype=np.float64)[active]
        Hl, Ll, Al, Gl = head_eval(hl, gammas[l], betas[l], Ws[l], eps, bf16)
        H[l, active], lse[l, active], am[l, active], gap[l, active] = Hl, Ll, Al, Gl
        still = []
        for pos, r in enumerate(active):
            leaves = (l == n_heads - 1) or (Hl[pos] < tau[l])
            if leaves:
                exit_layer[r] = l
                token[r] = Al[pos]
            else:
                still.append(r)
        active = np.asarray(still, dtype=np.int64)
    return dict(exit_layer=exit_layer, token=token, H=H, lse=lse, argmax=am,
                gap=gap, active=actives)


# ----------------------------------------------------------------------------
# DSSD greedy verification
# ----------------------------------------------------------------------------
def accepted_prefix(draft_row, target_row, length) -> int:
    """Largest n <= length with draft[j] == target[j] for every j < n."""
    n = 0
    while n < length and int(draft_row[n]) == int(target_row[n]):
        n += 1
    return n


def dssd_verify(f_final, draft, gamma, beta, W, draft_len=None, eps=1e-5, bf16=False):
    """Greedy verification of drafted tokens against the full model.

    f_final [B, k+1, d]: the full model's final hidden state at the position
    preceding each draft token (j = 0..k-1) plus the one after the last draft
    (j = k); draft [B, k].  target[b, j] is the final head's argmax on
    f_final[b, j]; accepted[b] is the length of the longest matching prefix
    (bounded by draft_len[b]); next_token[b] = target[b, accepted[b]] is the
    token written at the first mismatch, or the bonus token when every draft
    token is accepted.  Returns (accepted, next_token, target, gap).
    """
    f = np.asarray(f_final, dtype=np.float64)
    B, k1, d = f.shape
    k = k1 - 1
    draft = np.asarray(draft)
    _, _, am, gap = head_eval(f.reshape(B * k1, d), gamma, beta, W, eps, bf16)
    target = am.reshape(B, k1)
    gap = gap.reshape(B, k1)
    accepted = np.zeros(B, dtype=np.int64)
    nxt = np.zeros(B, dtype=np.int64)
    for b in range(B):
        L = k if draft_len is None else int(draft_len[b])
        accepted[b] = accepted_prefix(draft[b], target[b], L)
        nxt[b] = target[b, accepted[b]]
    return accepted, nxt, target, gap


def dssd_draft(H_by_position, token_by_position, tau, limit: int, eos_token: int):
    """Drafting phase of DSSD (Section 4.3.1) given, for every position the backbone
    can reach, the entropies H[t][l] and predictions token[t][l] of all heads
    (l = n_heads-1 is the full model's own head, which is no exit head).

    Walks the positions in order.  At position t the exit heads are tried from the
    shallowest to the deepest; the first with H < tau_l drafts its token: it is
    appended to the buffer.  Drafting stops (i) when the buffer holds `limit`
    tokens, (ii) right after an end-of-sequence token was appended, (iii) at a
    position where no exit head is confident: nothing is appended and the full
    model's prediction there is reported as the fallback token.  A NaN entropy is
    never under a threshold.  If the positions run out first the draft simply ends.

    Returns dict(draft, exit_layer (per drafted token), reason, fallback_token,
    n_evals) with reason in {"limit", "eos", "fallback", "exhausted"}; n_evals
    counts (position, head) evaluations with heads tried in order and the model's
    head evaluated at a fallback position.
    """
    n_heads = len(tau)
    draft, layers = [], []
    n_evals = 0
    reason, fallback = "exhausted", -1
    if limit <= 0:
        return dict(draft=draft, exit_layer=layers, reason="limit", fallback_token=-1, n_evals=0)
    for t in range(len(H_by_position)):
        chosen = None
        for l in range(n_heads - 1):
            n_evals += 1
            if H_by_position[t][l] < tau[l]:
                chosen = l
                break
        if chosen is None:
            n_evals += 1                          # the model's own head answers
            reason, fallback = "fallback", int(token_by_position[t][n_heads - 1])
            break
        tok = int(token_by_position[t][chosen])
        draft.append(tok)
        layers.append(chosen)
        if tok == eos_token:
            reason = "eos"
            break
        if len(draft) == limit:
            reason = "limit"
            break
    return dict(draft=draft, exit_layer=layers, reason=reason, fallback_token=fallback, n_evals=n_evals)


def dssd_tally(draft_len, accepted, exit_layers=None):
    """Bookkeeping over verification rounds (Section 4.3.1, verification phase, and the
    quantities Section 4.3.2 reports): every round b drafted draft_len[b] tokens of
    which the first accepted[b] were committed; the rest were computed for nothing.

    Returns dict(rounds, drafted, accepted, wasted, exit_layer_sum, acceptance_rate,
    mean_accepted) where acceptance_rate = accepted / drafted (NaN if nothing was
    drafted), mean_accepted = accepted / rounds (the "implicit speculation budget"),
    and exit_layer_sum adds exit_layers[b][j] over the drafted tokens j < draft_len[b]
    (0 without exit_layers), so that exit_layer_sum / drafted is the mean exit head
    during drafting.
    """
    rounds = drafted = acc = waste = layer_sum = 0
    for b in range(len(draft_len)):
        n, a = int(draft_len[b]), int(accepted[b])
        rounds += 1
        drafted += n
        acc += a
        waste += n - a
        if exit_layers is not None:
            for j in range(n):
                layer_sum += int(exit_layers[b][j])
    return dict(rounds=rounds, drafted=drafted, accepted=acc, wasted=waste, exit_layer_sum=layer_sum,
                acceptance_rate=acc / drafted if drafted else float("nan"),
                mean_accepted=acc / rounds if rounds else float("nan"))


# ----------------------------------------------------------------------------
# Training objectives, forward only (Section 3.3, "Losses")
# ----------------------------------------------------------------------------
def token_losses(z_head, z_model, labels=None):
    """Per-token loss terms of Section 3.3 from materialised logits.

    y_hat = softmax(z_head) is the exit head's distribution and f = softmax(z_model)
    the main model's.  For every token t:
      kl[t] = sum_v y_hat_v * log(y_hat_v / f_v)      (the head's distribution comes first,
                                                       as in the section's L_KL(y_hat || f_theta))
      ce[t] = -log y_hat_{labels[t]}                  (NaN without labels)
    Log-probabilities are taken as z - lse so that a vanishing probability contributes
    0 * finite = 0 (the 0 log 0 = 0 convention) instead of 0 * inf.  Returns (kl, ce).
    """
    zs = np.asarray(z_head, dtype=np.float64)
    zt = np.asarray(z_model, dtype=np.float64)
    if zs.ndim == 1:
        zs, zt = zs[None, :], zt[None, :]
    L = zs.shape[0]
    kl = np.empty(L)
    ce = np.full(L, np.nan)
    for t in range(L):
        ms, mt = zs[t].max(), zt[t].max()
        if not (np.isfinite(ms) and np.isfinite(mt)):
            kl[t] = np.nan
            continue
        logp = zs[t] - (ms + np.log(np.exp(zs[t] - ms).sum()))     # log y_hat
        logq = zt[t] - (mt + np.log(np.exp(zt[t] - mt).sum()))     # log f
        kl[t] = (np.exp(logp) * (logp - logq)).sum()
        if labels is not None:
            ce[t] = -logp[int(labels[t])]
    return kl, ce


def head_losses(h_head, h_model, gamma_head, beta_head, W_head, gamma_model, beta_model, W_model,
                labels=None, alpha=0.5, eps=1e-5, bf16=False):
    """The three training objectives of Section 3.3 for one exit head on a sequence of
    L tokens: both heads are LayerNorm -> projection (Section 3.2) on their own hidden
    states, h_head [L, d] from the head's block and h_model [L, d] from the last.

    L_CE = (1/L) sum_t ce[t]; L_KL = (1/L) sum_t kl[t]; L_hyb = alpha L_CE + (1 - alpha) L_KL.
    Returns dict(kl[L], ce[L], L_kl, L_ce, L_hyb); the CE terms are NaN without labels.
    """
    zs = head_logits(layernorm(h_head, gamma_head, beta_head, eps, bf16_out=bf16), W_head)
    zt = head_logits(layernorm(h_model, gamma_model, beta_model, eps, bf16_out=bf16), W_model)
    kl, ce = token_losses(zs, zt, labels)
    L = kl.shape[0]
    L_kl = kl.sum() / L if L else float("nan")
    L_ce = ce.sum() / L if L else float("nan")
    return dict(kl=kl, ce=ce, L_kl=L_kl, L_ce=L_ce, L_hyb=alpha * L_ce + (1.0 - alpha) * L_kl)


# ----------------------------------------------------------------------------
# Threshold calibration (Section 3.4.1, "Calibration of Confidence Thresholds")
# ----------------------------------------------------------------------------
def correctness(pred_head, pred_model) -> np.ndarray:
    """eq. (2): t_j = 1 where the head's prediction equals the underlying
    model's prediction for the same token, else 0."""
    return (np.asarray(pred_head) == np.asarray(pred_model)).astype(np.int64)


def calibrate_threshold(H, t, epsilon: float):
    """Entropy threshold of one head for the confidence level epsilon.

    The confidence is c = -H (a prediction is the more confident the lower its
    entropy).  Following Section 3.4.1 literally: take every calibration sample
    j in turn as the candidate threshold, look at ALL samples whose confidence
    is at least c_j (entropy at most H_j), and compute the proportion of
    correct predictions among them; among the candidates whose proportion is at
    least epsilon take the one that comes first in ascending order of
    confidence, i.e. the largest entropy.  tau is that sample's entropy.

    Readings: (i) the suffix of a candidate holds every sample with confidence
    "higher (or equal)", so samples tied with the candidate are all in it and
    the result does not depend on how ties are ordered; (ii) if no candidate
    qualifies the head never exits: tau = -inf; (iii) a NaN entropy is no
    candidate and belongs to no suffix (such a row never passes the exit test);
    (iv) the proportion test is the section's own expression, the quotient
    correct / size compared with epsilon, the quotient being the correctly rounded
    double (IEEE division): a proportion of exactly p/q therefore meets a level
    written as the decimal p/q (7 of 10 at 0.7, 11 of 20 at 0.55), which a product
    epsilon * size rounded to double does not guarantee.

    Quadratic on purpose (two nested sweeps, no sort, no running sums).
    Returns (tau, n) with n the number of samples with H <= tau.
    """
    H = np.asarray(H, dtype=np.float64)
    t = np.asarray(t)
    level = float(epsilon)
    best_H, best_n = -np.inf, 0
    for j in range(H.shape[0]):
        if np.isnan(H[j]):
            continue
        inside = H <= H[j]                       # NaN compares false: never inside
        size = int(np.count_nonzero(inside))
        correct = int(np.count_nonzero(t[inside]))
        if correct / size >= level and H[j] > best_H:
            best_H, best_n = float(H[j]), size
    return best_H, best_n
