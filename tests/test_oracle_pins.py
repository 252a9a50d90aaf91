"""Pins for the CPU oracle: what the paper's equations and plain mathematics fix.

None of these tests touches the GPU library.  Each one checks the oracle
against something other than itself: brute force in 50-digit arithmetic,
closed forms stored under tests/golden/ (written by make_closed_forms.py,
which never calls the oracle), scipy routines, invariances, and finite
differences.
"""
import math
import os

import mpmath
import numpy as np
import pytest
import scipy.special

from oracle import oapl_oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "closed_forms.txt")


def _golden(kind):
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            if parts[0] == kind:
                rows.append(parts[1:])
    assert rows, kind
    return rows


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- soft-max --

@pytest.mark.parametrize("V", [2, 3, 5, 17])
@pytest.mark.parametrize("d", [1, 3])
def test_logprob_brute_force_tiny_vocab(V, d):
    """Direct exp / sum without any max shift, in 50-digit arithmetic."""
    rng = _rng(100 * V + d)
    T = 6
    H = rng.normal(size=(T, d))
    W = rng.normal(size=(V, d))
    tok = rng.integers(0, V, size=T)
    lp, lse = orc.token_logprobs(H, W, tok)
    with mpmath.workdps(50):
        for t in range(T):
            z = [sum(mpmath.mpf(H[t, k]) * mpmath.mpf(W[v, k]) for k in range(d)) for v in range(V)]
            denom = sum(mpmath.exp(zv) for zv in z)
            want = mpmath.log(mpmath.exp(z[tok[t]]) / denom)
            assert abs(lp[t] - float(want)) < 1e-13
            assert abs(lse[t] - float(mpmath.log(denom))) < 1e-13


def test_zero_weights_give_minus_ln_vocab():
    for V, text in _golden("ln_vocab"):
        V = int(V)
        if V > 2048:
            T, d = 3, 4
        else:
            T, d = 9, 8
        H = _rng(V).normal(size=(T, d))
        W = np.zeros((V, d))
        tok = _rng(V + 1).integers(0, V, size=T)
        lp, lse = orc.token_logprobs(H, W, tok)
        assert np.allclose(lp, -float(text), rtol=0, atol=1e-14)
        assert np.allclose(lse, float(text), rtol=0, atol=1e-14)


def test_probabilities_sum_to_one_and_logprob_nonpositive():
    rng = _rng(7)
    T, d, V = 5, 6, 33
    H = rng.normal(size=(T, d)) * 3
    W = rng.normal(size=(V, d))
    total = np.zeros(T)
    for v in range(V):
        lp, _ = orc.token_logprobs(H, W, np.full(T, v))
        assert np.all(lp <= 0)
        total += np.exp(lp)
    assert np.allclose(total, 1.0, atol=1e-13)


def test_shift_invariance_of_weights():
    """Adding one vector u to every row of W shifts all logits of a row equally."""
    rng = _rng(8)
    T, d, V = 7, 5, 19
    H, W = rng.normal(size=(T, d)), rng.normal(size=(V, d))
    tok = rng.integers(0, V, size=T)
    u = rng.normal(size=d)
    lp0, lse0 = orc.token_logprobs(H, W, tok)
    lp1, lse1 = orc.token_logprobs(H, W + u, tok)
    assert np.allclose(lp0, lp1, atol=1e-12)
    assert np.allclose(lse1 - lse0, H @ u, atol=1e-12)


def test_vocab_permutation_with_relabelled_tokens():
    rng = _rng(9)
    T, d, V = 8, 4, 23
    H, W = rng.normal(size=(T, d)), rng.normal(size=(V, d))
    tok = rng.integers(0, V, size=T)
    perm = rng.permutation(V)          # new row j holds old row perm[j]
    inv = np.argsort(perm)
    lp0, _ = orc.token_logprobs(H, W, tok)
    lp1, _ = orc.token_logprobs(H, W[perm], inv[tok])
    assert np.allclose(lp0, lp1, atol=1e-13)


def test_matches_scipy_log_softmax():
    rng = _rng(10)
    T, d, V = 40, 16, 257
    H, W = rng.normal(size=(T, d)), rng.normal(size=(V, d))
    tok = rng.integers(0, V, size=T)
    lp, lse = orc.token_logprobs(H, W, tok, slab=7)   # slab must not matter
    ref = scipy.special.log_softmax(H @ W.T, axis=1)
    assert np.allclose(lp, ref[np.arange(T), tok], atol=1e-13)
    assert np.allclose(lse, scipy.special.logsumexp(H @ W.T, axis=1), atol=1e-13)


def test_row_selection_and_transposed_operand_mistakes_are_visible():
    """rows= picks rows of H (not of W); logits are H W^T, not H^T W."""
    rng = _rng(11)
    T, d, V = 12, 3, 12           # T == V on purpose: a transposed operand still has a legal shape
    H, W = rng.normal(size=(T, d)), rng.normal(size=(V, d))
    tok = rng.integers(0, V, size=T)
    rows = np.array([11, 0, 5])
    lp_all, _ = orc.token_logprobs(H, W, tok)
    lp_sel, _ = orc.token_logprobs(H, W, tok, rows=rows)
    assert np.array_equal(lp_all[rows], lp_sel)
    z = orc.logits(H, W)
    for t in range(T):
        for v in range(V):
            assert abs(z[t, v] - sum(H[t, k] * W[v, k] for k in range(d))) < 1e-13


def test_large_logits_do_not_overflow():
    rng = _rng(12)
    T, d, V = 4, 8, 50
    H, W = rng.normal(size=(T, d)) * 30, rng.normal(size=(V, d)) * 30
    tok = rng.integers(0, V, size=T)
    lp, lse = orc.token_logprobs(H, W, tok)
    assert np.all(np.isfinite(lp)) and np.all(np.isfinite(lse)) and np.all(lp <= 0)
    with mpmath.workdps(50):
        z = [mpmath.mpf(x) for x in (H[0] @ W.T)]
        want = z[tok[0]] - mpmath.log(sum(mpmath.exp(x) for x in z))
    assert abs(lp[0] - float(want)) < 1e-9 * max(1.0, abs(float(want)))


def test_integer_inputs_gather_is_exact():
    """Integer H, W make every logit an exact integer: lp + lse must return it."""
    rng = _rng(13)
    T, d, V = 30, 16, 64
    H = rng.integers(-2, 3, size=(T, d)).astype(np.float64)
    W = rng.integers(-2, 3, size=(V, d)).astype(np.float64)
    tok = rng.integers(0, V, size=T)
    lp, lse = orc.token_logprobs(H, W, tok)
    zy = np.array([int(H[t] @ W[tok[t]]) for t in range(T)], dtype=np.float64)
    assert np.allclose(lp + lse, zy, atol=1e-12)
    # a gather at the wrong index (tok[t] +- 1) would change most of these
    wrong = np.array([H[t] @ W[(tok[t] + 1) % V] for t in range(T)])
    assert np.abs(wrong - zy).max() >= 1.0


def test_token_out_of_range_is_an_error():
    H, W = np.ones((2, 2)), np.ones((3, 2))
    with pytest.raises(ValueError):
        orc.token_logprobs(H, W, np.array([0, 3]))
    with pytest.raises(ValueError):
        orc.token_logprobs(H, W, np.array([-1, 0]))


# ---------------------------------------------------------------- entropy --

def test_entropy_uniform_is_ln_vocab_and_bounds():
    for V, text in _golden("ln_vocab"):
        V = int(V)
        H = _rng(V).normal(size=(3, 4))
        ent = orc.token_entropy(H, np.zeros((V, 4)))
        assert np.allclose(ent, float(text), rtol=0, atol=1e-12)
    rng = _rng(70)
    H, W = rng.normal(size=(20, 6)) * 3, rng.normal(size=(41, 6))
    ent = orc.token_entropy(H, W)
    assert np.all(ent >= 0) and np.all(ent <= math.log(41) + 1e-12)


def test_entropy_brute_force_and_scipy():
    import scipy.stats
    rng = _rng(71)
    T, d, V = 7, 3, 9
    H, W = rng.normal(size=(T, d)) * 2, rng.normal(size=(V, d))
    ent = orc.token_entropy(H, W, slab=2)
    z = H @ W.T
    assert np.allclose(ent, scipy.stats.entropy(scipy.special.softmax(z, axis=1), axis=1), atol=1e-13)
    with mpmath.workdps(50):
        for t in range(T):
            e = [mpmath.exp(mpmath.mpf(x)) for x in z[t]]
            tot = sum(e)
            want = -sum((x / tot) * mpmath.log(x / tot) for x in e)
            assert abs(ent[t] - float(want)) < 1e-13
    # adding a vector to every row of W shifts all logits of a row equally: same distribution
    assert np.allclose(orc.token_entropy(H, W + rng.normal(size=d)), ent, atol=1e-12)
    # a nearly one-hot row has nearly zero entropy; rows= selects rows of H
    Hp = H.copy()
    Hp[2] *= 400
    e2 = orc.token_entropy(Hp, W, rows=np.array([2, 0]))
    assert e2[0] < 1e-6 and e2[1] == pytest.approx(ent[0], abs=1e-13)


# ---------------------------------------------------------------- sampling --

def test_philox_known_answers():
    """Known-answer vectors published with the generator (Random123 kat_vectors, philox4x32 10)."""
    kat = [
        ((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
        ((0xffffffff,) * 4, (0xffffffff,) * 2, (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
        ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
         (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1)),
    ]
    for ctr, key, want in kat:
        got = orc.philox4x32_10(np.array(ctr, dtype=np.uint32), np.array(key, dtype=np.uint32))
        assert tuple(int(x) for x in got) == want
    # vectorised call = element-wise call
    c = np.array([k[0] for k in kat], dtype=np.uint32)
    k = np.array([k[1] for k in kat], dtype=np.uint32)
    assert np.array_equal(orc.philox4x32_10(c, k), np.array([k_[2] for k_ in kat], dtype=np.uint32))


def test_gumbel_noise_layout_and_range():
    g = orc.gumbel_noise(np.array([0, 5, 2 ** 33 + 1]), 10, seed=(7 << 32) | 3)
    assert g.shape == (3, 10) and np.all(np.isfinite(g))
    # word v % 4 of the block with counter (v // 4, t_lo, t_hi, 0) and key (seed_lo, seed_hi)
    x = orc.philox4x32_10(np.array([2, 1, 2, 0], dtype=np.uint32), np.array([3, 7], dtype=np.uint32))
    u = ((int(x[1]) >> 9) + 0.5) * 2.0 ** -23
    assert g[2, 9] == -np.log(-np.log(u))
    # different rows, seeds and columns give different noise; the same arguments the same noise
    assert not np.array_equal(g[0], g[1])
    assert np.array_equal(orc.gumbel_noise(np.array([5]), 10, seed=(7 << 32) | 3)[0], g[1])
    assert not np.array_equal(orc.gumbel_noise(np.array([5]), 10, seed=4)[0], g[1])
    # standard Gumbel: mean = Euler's constant, variance = pi^2 / 6
    big = orc.gumbel_noise(np.arange(64), 4096, seed=11).ravel()
    assert abs(big.mean() - 0.5772156649) < 0.01 and abs(big.var() - np.pi ** 2 / 6) < 0.03


def test_sampled_tokens_follow_the_softmax():
    """Frequencies over many rows with identical hidden state match softmax(z / temperature)."""
    rng = _rng(80)
    d, V, n = 4, 6, 40000
    h = rng.normal(size=d)
    W = rng.normal(size=(V, d))
    H = np.tile(h, (n, 1))
    for temp in (1.0, 0.6):
        tok, best = orc.sample_tokens(H, W, temp, seed=123)
        p = scipy.special.softmax((W @ h) / temp)
        freq = np.bincount(tok, minlength=V) / n
        assert np.abs(freq - p).max() < 4 * np.sqrt(p.max() / n) + 1e-3
        # the reported score is the winner's perturbed logit, and it is the row maximum
        g = orc.gumbel_noise(np.arange(3), V, 123)
        s3 = (W @ h) / temp + g
        assert np.allclose(best[:3], s3.max(axis=1)) and np.array_equal(tok[:3], s3.argmax(axis=1))
    # rows= selects token rows: the draw depends on the row index, not on its position in the call
    t2, _ = orc.sample_tokens(H, W, 1.0, seed=123, rows=np.array([17, 3]))
    t0, _ = orc.sample_tokens(H, W, 1.0, seed=123)
    assert t2.tolist() == [t0[17], t0[3]]
    with pytest.raises(ValueError):
        orc.sample_tokens(H, W, 0.0, seed=1)


# ------------------------------------------------------- sequence log-ratio --

def test_sequence_logratio_exact_on_integers_and_empty_sequences():
    rng = _rng(20)
    off = np.array([0, 0, 1, 1, 9, 40, 40, 64])
    T = off[-1]
    lp = rng.integers(-9, 0, size=T).astype(np.float64)
    q = rng.integers(-9, 0, size=T).astype(np.float64)
    got = orc.sequence_logratio(lp, q, off)
    want = [sum(int(lp[t]) - int(q[t]) for t in range(off[s], off[s + 1])) for s in range(len(off) - 1)]
    assert got.tolist() == [float(w) for w in want]
    assert got[0] == 0.0 and got[2] == 0.0 and got[5] == 0.0


def test_sequence_logratio_sign_and_no_length_normalisation():
    lp = np.array([-1.0, -2.0, -3.0])
    q = np.array([-1.5, -1.5, -1.5])
    got = orc.sequence_logratio(lp, q, np.array([0, 3]))
    assert got[0] == pytest.approx(-6.0 + 4.5)          # sum of (lp - q), not mean, not (q - lp)


@pytest.mark.parametrize("off", [[1, 3], [0, 2], [0, 2, 1, 3], []])
def test_bad_offsets_are_errors(off):
    with pytest.raises(ValueError):
        orc.sequence_logratio(np.zeros(3), np.zeros(3), np.array(off, dtype=np.int64))


# ---------------------------------------------------- group value estimate --

def test_vstar_all_equal_rewards_is_the_reward_exactly():
    for r in (0.0, 1.0, 0.25, -3.5):
        for beta in (1e-3, 0.5, 1.0, 5.0):
            for G in (1, 4, 8, 16):
                v = orc.group_value_estimate(np.full(G, r), np.zeros(G, int), 1, beta)
                assert v[0] == r


def test_vstar_single_rollout_is_its_reward():
    v = orc.group_value_estimate(np.array([0.7, -0.2]), np.array([1, 0]), 2, 0.3)
    assert v.tolist() == [-0.2, 0.7]


def test_vstar_binary_closed_form():
    for G, k, beta, text in _golden("vstar_binary"):
        G, k, beta = int(G), int(k), float(beta)
        r = np.array([1.0] * k + [0.0] * (G - k))
        v = orc.group_value_estimate(r, np.zeros(G, int), 1, beta)
        assert v[0] == pytest.approx(float(text), rel=1e-15, abs=1e-16)


def test_vstar_limits_max_and_mean():
    """beta -> 0 gives the max reward, beta -> infinity the mean (Sec. 3.1)."""
    rng = _rng(30)
    r = rng.random(8)
    lo = orc.group_value_estimate(r, np.zeros(8, int), 1, 1e-4)[0]
    hi = orc.group_value_estimate(r, np.zeros(8, int), 1, 1e6)[0]
    assert abs(lo - r.max()) < 8 * 1e-4          # within beta * ln G of the max
    assert lo <= r.max()
    assert abs(hi - r.mean()) < 1e-6
    assert hi >= r.mean()                          # Jensen: the estimate is never below the mean


def test_vstar_matches_scipy_logsumexp_and_group_bookkeeping():
    rng = _rng(31)
    n, P = 37, 5
    gid = rng.integers(0, P, size=n)
    gid[:P] = np.arange(P)                          # every group non-empty
    r = rng.normal(size=n)
    for beta in (0.05, 1.0, 7.0):
        v = orc.group_value_estimate(r, gid, P, beta)
        for g in range(P):
            rg = r[gid == g]
            want = beta * (scipy.special.logsumexp(rg / beta) - math.log(rg.size))
            assert v[g] == pytest.approx(want, rel=1e-13, abs=1e-13)


def test_vstar_errors():
    with pytest.raises(ValueError):
        orc.group_value_estimate(np.ones(2), np.array([0, 0]), 2, 1.0)     # group 1 empty
    with pytest.raises(ValueError):
        orc.group_value_estimate(np.ones(2), np.array([0, 2]), 2, 1.0)     # id out of range
    with pytest.raises(ValueError):
        orc.group_value_estimate(np.ones(2), np.array([0, 1]), 2, 0.0)     # beta


# ------------------------------------------------------------------- loss --

def test_loss_on_policy_closed_form():
    """pi = pi_vllm: every log-ratio is 0, L = k (1 - V)^2 + (G - k) V^2."""
    for G, k, beta, text in _golden("loss_onpolicy"):
        G, k, beta = int(G), int(k), float(beta)
        r = np.array([1.0] * k + [0.0] * (G - k))
        loss, delta, _ = orc.oapl_loss(np.zeros(G), r, np.zeros(G, int), 1, beta)
        assert loss == pytest.approx(float(text), rel=1e-14, abs=1e-15)


def test_loss_residual_sign_and_beta_placement():
    # one prompt, two rollouts, rewards (1, 0), beta = 2
    beta = 2.0
    v = beta * math.log(0.5 * (math.exp(0.5) + 1.0))
    Delta = np.array([0.3, -0.1])
    loss, delta, vstar = orc.oapl_loss(Delta, np.array([1.0, 0.0]), np.array([0, 0]), 1, beta)
    assert vstar[0] == pytest.approx(v, rel=1e-15)
    assert delta[0] == pytest.approx(beta * 0.3 - (1.0 - v), rel=1e-14)
    assert delta[1] == pytest.approx(beta * -0.1 - (0.0 - v), rel=1e-14)
    assert loss == pytest.approx(delta[0] ** 2 + delta[1] ** 2, rel=1e-15)
    # two betas: beta_value only moves V*, beta only scales the log-ratio
    loss2, delta2, vstar2 = orc.oapl_loss(Delta, np.array([1.0, 0.0]), np.array([0, 0]), 1, 0.5, beta_value=2.0)
    assert vstar2[0] == pytest.approx(v, rel=1e-15)
    assert delta2[0] == pytest.approx(0.5 * 0.3 - (1.0 - v), rel=1e-14)
    # loss_scale multiplies the sum
    loss3, _, _ = orc.oapl_loss(Delta, np.array([1.0, 0.0]), np.array([0, 0]), 1, beta, loss_scale=0.25)
    assert loss3 == pytest.approx(0.25 * loss, rel=1e-15)


def _tiny_problem(seed, T_per=(3, 0, 4, 2, 1, 2), d=3, V=7, P=2):
    rng = _rng(seed)
    lens = np.array(T_per)
    off = np.concatenate([[0], np.cumsum(lens)])
    T = int(off[-1])
    H = rng.normal(size=(T, d))
    W = rng.normal(size=(V, d))
    tok = rng.integers(0, V, size=T)
    logq = -np.abs(rng.normal(size=T)) - 1.0
    n = lens.size
    gid = np.arange(n) % P
    rewards = (rng.random(n) < 0.5).astype(np.float64)
    return H, W, tok, logq, off, rewards, gid, P


def test_loss_invariant_under_sequence_permutation():
    H, W, tok, logq, off, r, gid, P = _tiny_problem(40)
    lp, _ = orc.token_logprobs(H, W, tok)
    Delta = orc.sequence_logratio(lp, logq, off)
    loss0, _, _ = orc.oapl_loss(Delta, r, gid, P, 0.7)
    perm = _rng(41).permutation(len(r))
    loss1, _, _ = orc.oapl_loss(Delta[perm], r[perm], gid[perm], P, 0.7)
    assert loss1 == pytest.approx(loss0, rel=1e-14)
    # relabelling the groups changes nothing either
    loss2, _, _ = orc.oapl_loss(Delta, r, (P - 1) - gid, P, 0.7)
    assert loss2 == pytest.approx(loss0, rel=1e-14)


def test_constructed_minimiser_has_zero_loss_and_zero_gradient():
    """If beta ln(pi / pi_vllm) = r - V* for every rollout, Eq. 3 is 0 and stationary."""
    H, W, tok, _, off, r, gid, P = _tiny_problem(42, T_per=(3, 2, 4, 2))
    beta = 0.8
    lp, _ = orc.token_logprobs(H, W, tok)
    vstar = orc.group_value_estimate(r, gid, P, beta)
    logq = np.empty_like(lp)
    for s in range(len(r)):
        a, b = off[s], off[s + 1]
        logq[a:b] = lp[a:b] - (r[s] - vstar[gid[s]]) / (beta * (b - a))
    res = orc.oapl_forward_backward(H, W, tok, logq, off, r, gid, P, beta)
    assert res["loss"] < 1e-25
    assert np.abs(res["dH"]).max() < 1e-12 and np.abs(res["dW"]).max() < 1e-12


# --------------------------------------------------------------- gradient --

@pytest.mark.parametrize("seed,beta,beta_value,scale", [(50, 1.0, None, 1.0), (51, 0.4, 1.5, 0.5)])
def test_gradients_match_central_finite_differences(seed, beta, beta_value, scale):
    H, W, tok, logq, off, r, gid, P = _tiny_problem(seed)
    res = orc.oapl_forward_backward(H, W, tok, logq, off, r, gid, P, beta,
                                    beta_value=beta_value, loss_scale=scale)

    def loss_of(Hx, Wx):
        return orc.oapl_forward_backward(Hx, Wx, tok, logq, off, r, gid, P, beta, beta_value=beta_value,
                                         loss_scale=scale, backward=False)["loss"]

    h = 1e-6
    scale_ref = max(np.abs(res["dH"]).max(), np.abs(res["dW"]).max())
    for name, A in (("dH", H), ("dW", W)):
        for idx in np.ndindex(A.shape):
            Ap, Am = A.copy(), A.copy()
            Ap[idx] += h
            Am[idx] -= h
            if name == "dH":
                fd = (loss_of(Ap, W) - loss_of(Am, W)) / (2 * h)
            else:
                fd = (loss_of(H, Ap) - loss_of(H, Am)) / (2 * h)
            assert abs(fd - res[name][idx]) < 2e-7 * scale_ref, (name, idx, fd, res[name][idx])


def test_gradient_invariants():
    H, W, tok, logq, off, r, gid, P = _tiny_problem(60, T_per=(5, 3, 0, 6, 2, 4), d=4, V=11)
    res = orc.oapl_forward_backward(H, W, tok, logq, off, r, gid, P, 1.3)
    # sum_v dZ[t, v] = 0  =>  the columns of dW sum to zero
    assert np.abs(res["dW"].sum(axis=0)).max() < 1e-12
    # <dH, H> = <dW, W> = sum_t sum_v dZ[t, v] z[t, v]
    assert np.sum(res["dH"] * H) == pytest.approx(np.sum(res["dW"] * W), rel=1e-12)
    # token coefficients are 2 beta delta of the owning rollout; empty rollouts own none
    for s in range(len(r)):
        assert np.all(res["coeff"][off[s]:off[s + 1]] == 2 * 1.3 * res["delta"][s])
    # the row-wise gradient helper is the same formula
    rows = np.array([0, 7, 19])
    g = orc.grad_hidden_rows(H, W, tok, res["coeff"], rows)
    assert np.allclose(g, res["dH"][rows], atol=1e-14)
    # ... and so is the row-wise weight gradient (every vocabulary row, in one piece and summed over
    # two slabs of token rows, each with its own slice of the per-token inputs)
    vsel = np.array([0, 3, 10, 5])
    gw = orc.grad_weight_rows(H, W[vsel], vsel, tok, res["coeff"], res["lse"])
    assert np.allclose(gw, res["dW"][vsel], atol=1e-13)
    cut = 9
    gw2 = (orc.grad_weight_rows(H[:cut], W[vsel], vsel, tok[:cut], res["coeff"][:cut], res["lse"][:cut]) +
           orc.grad_weight_rows(H[cut:], W[vsel], vsel, tok[cut:], res["coeff"][cut:], res["lse"][cut:]))
    assert np.allclose(gw2, res["dW"][vsel], atol=1e-13)
    allv = np.arange(W.shape[0])
    assert np.allclose(orc.grad_weight_rows(H, W, allv, tok, res["coeff"], res["lse"]), res["dW"], atol=1e-13)
    # a dropped one-hot term or a sign slip would not survive this: rows of sampled tokens differ from the rest
    assert set(tok) & set(vsel)


def test_rollouts_with_zero_residual_get_zero_gradient():
    H, W, tok, logq, off, r, gid, P = _tiny_problem(61, T_per=(4, 3, 5, 2), d=3, V=6)
    beta = 1.0
    lp, _ = orc.token_logprobs(H, W, tok)
    vstar = orc.group_value_estimate(r, gid, P, beta)
    s = 2
    a, b = off[s], off[s + 1]
    logq[a:b] = lp[a:b] - (r[s] - vstar[gid[s]]) / (beta * (b - a))
    res = orc.oapl_forward_backward(H, W, tok, logq, off, r, gid, P, beta)
    assert abs(res["delta"][s]) < 1e-13
    assert np.abs(res["dH"][a:b]).max() < 1e-12
    others = np.r_[0:a, b:off[-1]]
    assert np.abs(res["dH"][others]).max() > 1e-3


# ------------------------------------------------------------------- GRPO --

def _grpo_problem(seed):
    H, W, tok, logq, off, r, gid, P = _tiny_problem(seed, T_per=(3, 2, 4, 0, 2, 3), d=3, V=7)
    r = np.array([1.0, 0.0, 0.0, 1.0, 1.0, 0.0])       # every group has both outcomes
    rng = _rng(seed + 1)
    lp, _ = orc.token_logprobs(H, W, tok)
    logp_old = lp + rng.normal(scale=0.1, size=lp.size)
    logq = logp_old + rng.normal(scale=0.1, size=lp.size)
    return H, W, tok, logq, logp_old, off, r, gid, P


def test_grpo_advantages_are_group_normalised():
    r = np.array([1.0, 0.0, 0.0, 1.0, 1.0, 0.0, 3.0])
    gid = np.array([0, 1, 0, 1, 0, 1, 1])
    A = orc.grpo_advantages(r, gid, 2, adv_eps=0.0)
    for g in (0, 1):
        a = A[gid == g]
        assert abs(a.mean()) < 1e-15 and abs((a ** 2).mean() - 1.0) < 1e-14      # population variance 1
    assert A[0] == pytest.approx((1 - 2 / 3) / math.sqrt(2 / 9))
    # all-equal rewards: zero advantage (the epsilon keeps 0 / 0 away)
    assert orc.grpo_advantages(np.ones(4), np.zeros(4, int), 1).tolist() == [0.0] * 4


def test_grpo_on_policy_closed_form():
    """pi = pi_old = pi_vllm: every ratio is 1, each non-empty rollout contributes A_i / G to the
    objective (so it is 0 when no rollout of a group is empty) and the coefficient of every token of
    rollout i is -A_i / (G |y_i|)."""
    H, W, tok, _, _, off, r, gid, P = _grpo_problem(90)
    lp, _ = orc.token_logprobs(H, W, tok)
    res = orc.grpo_forward_backward(H, W, tok, lp, lp, off, r, gid, P)
    A = orc.grpo_advantages(r, gid, P)
    G = np.bincount(gid, minlength=P)
    nonempty = np.diff(off) > 0
    assert res["loss"] == pytest.approx(-sum(A[s] / G[gid[s]] for s in range(len(r)) if nonempty[s]), rel=1e-13)
    # without the empty rollout the normalised advantages of each group cancel
    keep = np.nonzero(nonempty)[0]
    off2 = np.concatenate([[0], np.cumsum(np.diff(off)[keep])])
    res2 = orc.grpo_forward_backward(H, W, tok, lp, lp, off2, r[keep], gid[keep], P)
    assert abs(res2["loss"]) < 1e-14
    for s in range(len(r)):
        a, b = off[s], off[s + 1]
        if b > a:
            assert np.allclose(res["coeff"][a:b], -A[s] / (G[gid[s]] * (b - a)), rtol=1e-12)


def test_grpo_clipped_tokens_are_flat_and_unclipped_are_not():
    adv = np.array([2.0, 2.0, -2.0, -2.0, 2.0])
    lp_old = np.zeros(5)
    lp = np.log(np.array([1.5, 1.1, 0.5, 0.9, 0.7]))       # ratios r_t
    logq = np.full(5, np.log(0.5))                          # IS = pi_old / pi_vllm = 2
    term, dterm = orc.grpo_token_terms(lp, lp_old, logq, adv, 0.2)
    # A > 0, r > 1 + eps: clipped at 1.2 A;  A < 0, r < 1 - eps: clipped at 0.8 A;  others r A
    assert np.allclose(term, 2 * np.array([1.2 * 2, 1.1 * 2, 0.8 * -2, 0.9 * -2, 0.7 * 2]))
    assert np.allclose(dterm, 2 * np.array([0.0, 1.1 * 2, 0.0, 0.9 * -2, 0.7 * 2]))


@pytest.mark.parametrize("seed", [91, 92])
def test_grpo_gradients_match_finite_differences(seed):
    H, W, tok, logq, logp_old, off, r, gid, P = _grpo_problem(seed)
    res = orc.grpo_forward_backward(H, W, tok, logq, logp_old, off, r, gid, P, loss_scale=0.5)
    lp = res["logprob"]
    ratio = np.exp(lp - logp_old)
    assert np.abs(ratio - 1.2).min() > 1e-3 and np.abs(ratio - 0.8).min() > 1e-3     # away from the kinks

    def loss_of(Hx, Wx):
        return orc.grpo_forward_backward(Hx, Wx, tok, logq, logp_old, off, r, gid, P, loss_scale=0.5,
                                         backward=False)["loss"]
    h = 1e-6
    ref = max(np.abs(res["dH"]).max(), np.abs(res["dW"]).max())
    for name, A in (("dH", H), ("dW", W)):
        for idx in np.ndindex(A.shape):
            Ap, Am = A.copy(), A.copy()
            Ap[idx] += h
            Am[idx] -= h
            fd = (loss_of(Ap, W) - loss_of(Am, W)) / (2 * h) if name == "dH" else \
                 (loss_of(H, Ap) - loss_of(H, Am)) / (2 * h)
            assert abs(fd - res[name][idx]) < 2e-7 * ref + 1e-10, (name, idx, fd, res[name][idx])
    assert np.abs(res["dW"].sum(axis=0)).max() < 1e-13
