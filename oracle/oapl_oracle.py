"""CPU oracle for the OAPL trainer-step loss head (fp64, numpy).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow statement of what the
GPU library must compute.  It is imported by the tests, by the smoke check and
by the benchmark's CPU-baseline leg, and by nothing else; it shares no code,
tables or helpers with the HIP path and never calls it.

What it computes, in the paper's order and notation:

* the per-token log-probability of the sampled token under the trainer policy
  pi, ln pi(y_t | x, y_<t), with pi the soft-max over the full vocabulary of
  the LM-head logits z_t = W h_t at temperature 1 (Sec. 2; generation settings
  in the appendix use temperature 1 and top-p 1);
* the sequence log-ratio ln pi(y|x) - ln pi_vllm(y|x) as the plain sum over the
  rollout's tokens (Eq. 3 is written at sequence level and carries no length
  normalisation);
* the group value estimate V*(x) = beta ln (1/G) sum_i exp(r(x, y_i) / beta)
  (Sec. 3.1, Eq. 2);
* the OAPL objective sum_x sum_i (beta ln(pi/pi_vllm) - (r - V*))^2
  (Sec. 3.1, Eq. 3), a plain sum of squares with no ratios and no clipping;
* its gradient with respect to the hidden states H and the LM-head weights W
  by the chain rule, with V* and the inference log-probs held constant (V* is
  a function of rewards only).

All floating point is float64 except the value estimate, which evaluates
Eq. 2 literally in 50-digit arithmetic so that exp(r / beta) cannot overflow
for the small betas the paper's experiments use.  Dense contractions are
``numpy.matmul`` calls; rows are processed in slabs only to bound memory (every
token row is independent).  There is no tiling, no online merging and no
reordering of the definitions.

The per-token policy entropy (the training-stability diagnostic of Sec. 6.1)
is computed from the same log-soft-max.  The sampling step of Alg. 1 (draw
y_t from softmax(z_t / temperature)) is stated as a Gumbel-max draw over a
counter-based generator (Philox-4x32-10) so that a GPU kernel can reproduce
the same draws; it is pinned by the generator's published known-answer
vectors and by the draw frequencies matching the soft-max.  The paper's
baseline objective, GRPO with token-level importance sampling (Sec. 2), is
stated on the same log-probs; pins: zero loss and the closed-form gradient
coefficients when all three policies agree, flat clipped branches, and finite
differences.

Pins (tests/test_oracle_pins.py): brute-force soft-max on tiny vocabularies in
50-digit arithmetic, W = 0 giving -ln V, shift and permutation invariances,
scipy's log_softmax and logsumexp, the beta -> 0 / beta -> infinity limits of
Eq. 2, the all-equal-rewards closed form V* = r, the binary-reward closed form,
the pi = pi_vllm closed form of Eq. 3, the constructed minimiser of Eq. 3
(loss 0, gradient 0), central finite differences for every element of dH
and dW (the row-wise forms grad_hidden_rows / grad_weight_rows: equality with
those), and for the entropy: ln V for uniform logits, 50-digit brute force,
scipy.stats.entropy, the bounds 0 <= H <= ln V and shift invariance.  No
value the paper prints exists for this path (it prints no worked example), so
full-size numbers are pinned by these properties only.
"""
from __future__ import annotations

import math

import numpy as np
import mpmath

_MP_DIGITS = 50


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


# --------------------------------------------------------------------------
# Per-token log-probabilities (soft-max over the full vocabulary, Sec. 2)
# --------------------------------------------------------------------------

def logits(H, W) -> np.ndarray:
    """z[t, v] = sum_k H[t, k] W[v, k]."""
    return _f64(H) @ _f64(W).T


def log_softmax_rows(z: np.ndarray):
    """Two-pass log-soft-max of each row: returns (log p, lse)."""
    m = z.max(axis=1, keepdims=True)
    lse = m + np.log(np.exp(z - m).sum(axis=1, keepdims=True))
    return z - lse, lse[:, 0]


def token_logprobs(H, W, tokens, rows=None, slab: int = 256):
    """ln pi(y_t | .) and the log-partition lse_t for the selected token rows.

    ``rows`` (optional) is an index array into the packed token stream; the
    result is aligned with it.  Returns (lp, lse), both float64.
    """
    W64 = _f64(W)
    tokens = np.asarray(tokens).astype(np.int64)
    if rows is None:
        rows = np.arange(np.asarray(H).shape[0])
    rows = np.asarray(rows, dtype=np.int64)
    if tokens.size and (tokens[rows].min() < 0 or tokens[rows].max() >= W64.shape[0]):
        raise ValueError("sampled token outside [0, V)")
    lp = np.empty(rows.size, dtype=np.float64)
    lse = np.empty(rows.size, dtype=np.float64)
    for a in range(0, rows.size, slab):
        r = rows[a:a + slab]
        z = _f64(np.asarray(H)[r]) @ W64.T
        logp, l = log_softmax_rows(z)
        lp[a:a + r.size] = logp[np.arange(r.size), tokens[r]]
        lse[a:a + r.size] = l
    return lp, lse


def token_entropy(H, W, rows=None, slab: int = 256) -> np.ndarray:
    """Entropy of the trainer policy's next-token distribution, -sum_v p_v ln p_v, per token row.

    This is the quantity whose collapse (GRPO) or stability (OAPL) the paper's training-dynamics
    discussion tracks (Sec. 6.1).  Terms with p_v = 0 contribute 0.
    """
    W64 = _f64(W)
    Hn = np.asarray(H)
    if rows is None:
        rows = np.arange(Hn.shape[0])
    rows = np.asarray(rows, dtype=np.int64)
    out = np.empty(rows.size, dtype=np.float64)
    for a in range(0, rows.size, slab):
        r = rows[a:a + slab]
        logp, _ = log_softmax_rows(_f64(Hn[r]) @ W64.T)
        p = np.exp(logp)
        out[a:a + r.size] = -np.sum(np.where(p > 0, p * logp, 0.0), axis=1)
    return out


# --------------------------------------------------------------------------
# Sampling step of Alg. 1: y_t ~ softmax(z_t / temperature) by the Gumbel-max construction
# --------------------------------------------------------------------------

_PHILOX_M0, _PHILOX_M1 = 0xD2511F53, 0xCD9E8D57
_PHILOX_W0, _PHILOX_W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter, key):
    """Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
    as 1, 2, 3", SC'11), vectorised: counter [..., 4] and key [..., 2] uint32 -> [..., 4] uint32."""
    c = [np.asarray(counter)[..., i].astype(np.uint64) for i in range(4)]
    k0 = np.asarray(key)[..., 0].astype(np.uint64)
    k1 = np.asarray(key)[..., 1].astype(np.uint64)
    mask = np.uint64(0xFFFFFFFF)
    for _ in range(10):
        p0 = np.uint64(_PHILOX_M0) * c[0]
        p1 = np.uint64(_PHILOX_M1) * c[2]
        c = [(p1 >> np.uint64(32)) ^ c[1] ^ k0, p1 & mask, (p0 >> np.uint64(32)) ^ c[3] ^ k1, p0 & mask]
        k0 = (k0 + np.uint64(_PHILOX_W0)) & mask
        k1 = (k1 + np.uint64(_PHILOX_W1)) & mask
    return np.stack(c, axis=-1).astype(np.uint32)


def gumbel_noise(rows, V: int, seed: int) -> np.ndarray:
    """g[t, v] = -ln(-ln u[t, v]) for the given token rows, all v in [0, V).

    u comes from Philox-4x32-10 with key (seed low word, seed high word) and counter
    (v // 4, t low word, t high word, 0); output word v % 4 gives x, and
    u = ((x >> 9) + 1/2) * 2^-23, which lies strictly inside (0, 1) and is exact in binary32.
    """
    rows = np.asarray(rows, dtype=np.int64)
    nb = (V + 3) // 4
    ctr = np.zeros((rows.size, nb, 4), dtype=np.uint32)
    ctr[:, :, 0] = np.arange(nb, dtype=np.uint32)[None, :]
    ctr[:, :, 1] = (rows & 0xFFFFFFFF).astype(np.uint32)[:, None]
    ctr[:, :, 2] = (rows >> 32).astype(np.uint32)[:, None]
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    x = philox4x32_10(ctr, np.broadcast_to(key, ctr.shape[:-1] + (2,))).reshape(rows.size, nb * 4)[:, :V]
    u = ((x >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23
    return -np.log(-np.log(u))


def sample_tokens(H, W, temperature: float, seed: int, rows=None, slab: int = 128):
    """One draw per token row from softmax(z_t / temperature): argmax_v (z_tv / temperature + g_tv)
    (ties to the smallest v).  Returns (tokens, scores) where scores[t] is the winning perturbed logit.
    """
    if not temperature > 0:
        raise ValueError("temperature must be positive")
    W64 = _f64(W)
    Hn = np.asarray(H)
    V = W64.shape[0]
    if rows is None:
        rows = np.arange(Hn.shape[0])
    rows = np.asarray(rows, dtype=np.int64)
    tok = np.empty(rows.size, dtype=np.int64)
    best = np.empty(rows.size, dtype=np.float64)
    for a in range(0, rows.size, slab):
        r = rows[a:a + slab]
        score = (_f64(Hn[r]) @ W64.T) / float(temperature) + gumbel_noise(r, V, seed)
        tok[a:a + r.size] = np.argmax(score, axis=1)
        best[a:a + r.size] = score[np.arange(r.size), tok[a:a + r.size]]
    return tok, best


# --------------------------------------------------------------------------
# Sequence log-ratio (Eq. 3, the ln pi(y|x) / pi_vllm(y|x) term)
# --------------------------------------------------------------------------

def check_offsets(seq_offsets, T: int) -> np.ndarray:
    off = np.asarray(seq_offsets).astype(np.int64)
    if off.ndim != 1 or off.size < 1 or off[0] != 0 or off[-1] != T or np.any(np.diff(off) < 0):
        raise ValueError("seq_offsets must start at 0, end at T and be non-decreasing")
    return off


def sequence_logratio(lp, logq, seq_offsets) -> np.ndarray:
    """Delta_s = sum over the tokens of rollout s of (ln pi(y_t) - ln pi_vllm(y_t))."""
    lp = _f64(lp)
    logq = _f64(logq)
    off = check_offsets(seq_offsets, lp.shape[0])
    out = np.zeros(off.size - 1, dtype=np.float64)
    for s in range(off.size - 1):
        a, b = int(off[s]), int(off[s + 1])
        out[s] = float(np.sum(lp[a:b] - logq[a:b]))
    return out


# --------------------------------------------------------------------------
# Group value estimate (Eq. 2)
# --------------------------------------------------------------------------

def group_value_estimate(rewards, group_ids, n_groups: int, beta: float) -> np.ndarray:
    """V*(x) = beta ln( (1/G) sum_{i=1..G} exp(r(x, y_i) / beta) ) per prompt.

    Evaluated exactly as written, in 50-digit arithmetic.  G is the number of
    rollouts that carry the prompt's group id.
    """
    rewards = _f64(rewards)
    gid = np.asarray(group_ids).astype(np.int64)
    if beta <= 0 or not np.isfinite(beta):
        raise ValueError("beta must be positive and finite")
    if gid.size and (gid.min() < 0 or gid.max() >= n_groups):
        raise ValueError("group id outside [0, n_groups)")
    out = np.empty(n_groups, dtype=np.float64)
    with mpmath.workdps(_MP_DIGITS):
        b = mpmath.mpf(float(beta))
        for g in range(n_groups):
            r = rewards[gid == g]
            if r.size == 0:
                raise ValueError(f"group {g} has no rollouts")
            acc = mpmath.mpf(0)
            for ri in r:
                acc += mpmath.exp(mpmath.mpf(float(ri)) / b)
            out[g] = float(b * mpmath.log(acc / r.size))
    return out


# --------------------------------------------------------------------------
# Objective (Eq. 3) and its gradient
# --------------------------------------------------------------------------

def oapl_residuals(seq_logratio, rewards, group_ids, n_groups: int, beta: float,
                   beta_value: float | None = None):
    """delta_s = beta * Delta_s - (r_s - V*(x_s)).

    ``beta`` is the coefficient of Eq. 3.  ``beta_value`` is the coefficient of
    Eq. 2; it defaults to ``beta`` (the method section uses one constant; the
    experimental section allows two).
    Returns (delta, vstar).
    """
    vstar = group_value_estimate(rewards, group_ids, n_groups,
                                 beta if beta_value is None else beta_value)
    gid = np.asarray(group_ids).astype(np.int64)
    adv = _f64(rewards) - vstar[gid]
    delta = float(beta) * _f64(seq_logratio) - adv
    return delta, vstar


def oapl_loss(seq_logratio, rewards, group_ids, n_groups: int, beta: float,
              beta_value: float | None = None, loss_scale: float = 1.0):
    """Eq. 3: loss_scale * sum_s delta_s^2.  Returns (loss, delta, vstar)."""
    delta, vstar = oapl_residuals(seq_logratio, rewards, group_ids, n_groups, beta, beta_value)
    return float(loss_scale) * float(np.sum(delta * delta)), delta, vstar


def token_coefficients(delta, seq_offsets, beta: float, loss_scale: float = 1.0) -> np.ndarray:
    """c_t = dL / d ln pi(y_t) = loss_scale * 2 * beta * delta_{s(t)}."""
    off = np.asarray(seq_offsets).astype(np.int64)
    c = np.zeros(int(off[-1]), dtype=np.float64)
    for s in range(off.size - 1):
        c[int(off[s]):int(off[s + 1])] = float(loss_scale) * 2.0 * float(beta) * delta[s]
    return c


def grad_hidden_rows(H, W, tokens, coeff, rows, slab: int = 256) -> np.ndarray:
    """dL/dH for the selected rows: c_t * (W[y_t, :] - sum_v p_{t,v} W[v, :])."""
    W64 = _f64(W)
    tokens = np.asarray(tokens).astype(np.int64)
    rows = np.asarray(rows, dtype=np.int64)
    coeff = _f64(coeff)
    out = np.empty((rows.size, W64.shape[1]), dtype=np.float64)
    for a in range(0, rows.size, slab):
        r = rows[a:a + slab]
        z = _f64(np.asarray(H)[r]) @ W64.T
        logp, _ = log_softmax_rows(z)
        p = np.exp(logp)
        out[a:a + r.size] = coeff[r, None] * (W64[tokens[r]] - p @ W64)
    return out


def grad_weight_rows(H, W_rows, vocab_rows, tokens, coeff, lse) -> np.ndarray:
    """dL/dW for the selected vocabulary rows, from the token rows given:

        dW[v, :] = sum_t c_t * (1[v == y_t] - exp(z_{t,v} - lse_t)) * H[t, :],   z_{t,v} = W[v, :] . H[t, :]

    (chain rule on Eq. 3, with the soft-max written through the log-partition lse_t of each token
    row).  ``W_rows`` are the selected rows of W, ``vocab_rows`` their indices v.  The sum over t is
    linear: a caller that cannot hold all token rows at once adds up the results of slabs.
    """
    H64 = _f64(H)
    Wr = _f64(W_rows)
    vocab_rows = np.asarray(vocab_rows, dtype=np.int64)
    tokens = np.asarray(tokens).astype(np.int64)
    c = _f64(coeff)
    z = H64 @ Wr.T                                            # [t, selected v]
    g = -np.exp(z - _f64(lse)[:, None])
    g += (tokens[:, None] == vocab_rows[None, :])             # the one-hot term
    g *= c[:, None]
    return g.T @ H64


def oapl_forward_backward(H, W, tokens, logq, seq_offsets, rewards, group_ids,
                          n_groups: int, beta: float, beta_value: float | None = None,
                          loss_scale: float = 1.0, backward: bool = True, slab: int = 256):
    """The whole path on one batch.  Returns a dict of float64 results.

    keys: logprob [T], lse [T], seq_logratio [N], vstar [P], delta [N], loss,
    and with ``backward``: coeff [T], dH [T, d], dW [V, d].
    """
    H64 = _f64(H)
    W64 = _f64(W)
    T, d = H64.shape
    V = W64.shape[0]
    tokens = np.asarray(tokens).astype(np.int64)
    off = check_offsets(seq_offsets, T)

    lp, lse = token_logprobs(H64, W64, tokens, slab=slab)
    Delta = sequence_logratio(lp, logq, off)
    loss, delta, vstar = oapl_loss(Delta, rewards, group_ids, n_groups, beta, beta_value, loss_scale)
    res = dict(logprob=lp, lse=lse, seq_logratio=Delta, vstar=vstar, delta=delta, loss=loss)
    if not backward:
        return res

    c = token_coefficients(delta, off, beta, loss_scale)
    dH = np.empty((T, d), dtype=np.float64)
    dW = np.zeros((V, d), dtype=np.float64)
    for a in range(0, T, slab):
        b = min(T, a + slab)
        z = H64[a:b] @ W64.T
        p = np.exp(z - lse[a:b, None])
        # dL/dz[t, v] = c_t * (1[v == y_t] - p[t, v])
        dZ = -p
        dZ[np.arange(b - a), tokens[a:b]] += 1.0
        dZ *= c[a:b, None]
        dH[a:b] = dZ @ W64
        dW += dZ.T @ H64[a:b]
    res.update(coeff=c, dH=dH, dW=dW)
    return res


# --------------------------------------------------------------------------
# The paper's baseline objective on the same head: GRPO with token-level
# importance sampling (Sec. 2, the displayed GRPO equation)
# --------------------------------------------------------------------------

def grpo_advantages(rewards, group_ids, n_groups: int, adv_eps: float = 1e-6) -> np.ndarray:
    """Normalised advantage of each rollout inside its prompt's group:
    A_i = (r_i - mean_g r) / (std_g r + adv_eps), population standard deviation."""
    r = _f64(rewards)
    gid = np.asarray(group_ids).astype(np.int64)
    if gid.size and (gid.min() < 0 or gid.max() >= n_groups):
        raise ValueError("group id outside [0, n_groups)")
    A = np.empty_like(r)
    for g in range(n_groups):
        sel = gid == g
        if not sel.any():
            raise ValueError(f"group {g} has no rollouts")
        rg = r[sel]
        mean = rg.sum() / rg.size
        std = math.sqrt(((rg - mean) ** 2).sum() / rg.size)
        A[sel] = (rg - mean) / (std + adv_eps)
    return A


def grpo_token_terms(lp, logp_old, logq, adv_t, clip_eps: float):
    """Per token: IS_t * min(r_t A_t, clip(r_t, 1 - eps, 1 + eps) A_t) and its derivative with
    respect to ln pi(y_t), where r_t = pi / pi_old and IS_t = pi_old / pi_vllm."""
    r = np.exp(_f64(lp) - _f64(logp_old))
    w_is = np.exp(_f64(logp_old) - _f64(logq))
    unclipped = r * adv_t
    clipped = np.clip(r, 1.0 - clip_eps, 1.0 + clip_eps) * adv_t
    term = w_is * np.minimum(unclipped, clipped)
    dterm = np.where(unclipped <= clipped, w_is * unclipped, 0.0)    # d(r A)/d ln pi = r A; the clipped branch is flat
    return term, dterm


def grpo_forward_backward(H, W, tokens, logq, logp_old, seq_offsets, rewards, group_ids, n_groups: int,
                          clip_eps: float = 0.2, adv_eps: float = 1e-6, loss_scale: float = 1.0,
                          backward: bool = True, slab: int = 256):
    """loss = -loss_scale * sum_x (1/G_x) sum_{y in group x} (1/|y|) sum_t IS_t min(r_t A, clip(r_t) A)
    (the objective of Sec. 2 is maximised, so its negative is the loss; empty rollouts contribute 0)
    and its gradients with respect to H and W.  Returns a dict like oapl_forward_backward."""
    H64, W64 = _f64(H), _f64(W)
    T, d = H64.shape
    V = W64.shape[0]
    tokens = np.asarray(tokens).astype(np.int64)
    off = check_offsets(seq_offsets, T)
    gid = np.asarray(group_ids).astype(np.int64)
    lp, lse = token_logprobs(H64, W64, tokens, slab=slab)
    A = grpo_advantages(rewards, gid, n_groups, adv_eps)
    G = np.bincount(gid, minlength=n_groups).astype(np.float64)
    n_seq = off.size - 1
    loss = 0.0
    c = np.zeros(T, dtype=np.float64)
    for s_ in range(n_seq):
        a, b = int(off[s_]), int(off[s_ + 1])
        if b == a:
            continue
        term, dterm = grpo_token_terms(lp[a:b], _f64(logp_old)[a:b], _f64(logq)[a:b], A[s_], clip_eps)
        w = float(loss_scale) / (G[gid[s_]] * (b - a))
        loss -= w * float(term.sum())
        c[a:b] = -w * dterm
    res = dict(logprob=lp, lse=lse, advantages=A, loss=loss, coeff=c)
    if not backward:
        return res
    dH = np.empty((T, d), dtype=np.float64)
    dW = np.zeros((V, d), dtype=np.float64)
    for a in range(0, T, slab):
        b = min(T, a + slab)
        p = np.exp(H64[a:b] @ W64.T - lse[a:b, None])
        dZ = -p
        dZ[np.arange(b - a), tokens[a:b]] += 1.0
        dZ *= c[a:b, None]
        dH[a:b] = dZ @ W64
        dW += dZ.T @ H64[a:b]
    res.update(dH=dH, dW=dW)
    return res
