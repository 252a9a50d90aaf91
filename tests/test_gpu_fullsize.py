"""Full-size runs of the four bf16 configurations, in the launch configuration bench.py times
(default panel size, panel buffers for the workload's longest rollout, single sweep).

A full fp64 oracle pass is feasible for the forward-only configuration (2 T V d = 2e13 flop) and is
run there; for the others (6 T V d = 5e14 .. 4e15 flop) each configuration is checked in layers on
the same seeded inputs:

 (A) PARITY on outputs the oracle computes one by one:
     * per-token log-probs (and the log-partition of the forward entry point) at >= 4096 token rows:
       first and last token of every rollout, rows around token-tile and panel edges, random rows;
       their mean signed error bounds the bias a 32768-token sum could accumulate;
     * every token of complete rollouts (the shortest of each prompt, as many as ~6000 oracle rows
       allow): the rollout's log-ratio Delta_s, its residual delta_s and its share of the loss
       against the oracle's (the forward-only configuration: all rollouts, i.e. the full loss);
     * every group value estimate (they depend on rewards only);
     * rows of dH at the sampled token rows, and rows of dW at ~64 vocabulary rows (tile edges, the
       ragged last tile, rows of sampled tokens, random rows), the latter summed over ALL T token
       rows by the oracle's row formula -- a dropped or doubled panel cannot hide there.
 (B) PARITY of every output, element by element, on a 1024-token slice of the same configuration
     (same d, V, dtype, weights) that the oracle can do in full, also for the two-beta variant
     and the GRPO baseline.
 (C) PROPERTIES that hold at any size, checked on the full-size outputs (consistency checks, not
     parity claims): the per-rollout log-ratio equals the segment sum of the exported log-probs
     minus logq (every token -> rollout map exact), the loss equals the sum of squared residuals
     built from those log-ratios and the oracle's value estimates, the columns of dW sum to zero,
     <dH, H> = <dW, W>, and the gradients are finite.
"""
import time

import numpy as np
import pytest
import torch

from oracle import oapl_oracle as orc
from paper_2602_19362_amd import oapl
from workloads import synth
from tests._util import f64, grad_norm, rel

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
N_SAMPLED = 4096          # least number of token rows whose log-probs the oracle recomputes
ROLLOUT_ROW_BUDGET = 6000  # oracle rows spent on complete rollouts (configurations without a full oracle pass)


def _say(name, msg):
    print(f"[{name}] {msg}", flush=True)


def _sample_rows(off, T, panel_rows, n_total, seed):
    rows = set()
    for s in range(len(off) - 1):
        if off[s + 1] > off[s]:
            rows.add(int(off[s]))
            rows.add(int(off[s + 1] - 1))
    for edge in (0, 191, 192, 255, 256, 383, 384, 385, 767, 768, T - 385, T - 384, T - 1):   # token-tile edges
        if 0 <= edge < T:
            rows.add(int(edge))
    for k in range(1, T // panel_rows + 1):          # around every panel boundary of the plan in use
        for e in (k * panel_rows - 1, k * panel_rows, k * panel_rows + 1):
            if 0 <= e < T:
                rows.add(int(e))
    rng = np.random.default_rng(seed)
    while len(rows) < min(n_total, T):
        rows.update(int(x) for x in rng.integers(0, T, size=n_total - len(rows)))
    return np.array(sorted(rows), dtype=np.int64)


def _oracle_logprobs(name, b, W64, rows, what):
    """Oracle (lp, lse) at the given token rows, in chunks, saying how far it is."""
    lp = np.empty(rows.size)
    lse = np.empty(rows.size)
    t0 = time.time()
    for a in range(0, rows.size, 2048):
        r = rows[a:a + 2048]
        rt = torch.from_numpy(r).to(DEV)
        lp[a:a + r.size], lse[a:a + r.size] = orc.token_logprobs(f64(b.H[rt]), W64, b.tokens[rt].cpu().numpy())
        _say(name, f"oracle {what}: {min(a + 2048, rows.size)}/{rows.size} rows, {time.time() - t0:.0f} s")
    return lp, lse


def _complete_rollouts(off, gid, n_groups, budget):
    """The shortest non-empty rollout of each prompt, shortest first, while the row budget lasts."""
    lens = np.diff(off)
    picks = []
    for g in range(n_groups):
        cand = [s for s in range(lens.size) if gid[s] == g and lens[s] > 0]
        if cand:
            picks.append(min(cand, key=lambda s: lens[s]))
    picks.sort(key=lambda s: lens[s])
    out, used = [], 0
    for s in picks:
        if used + lens[s] <= budget:
            out.append(s)
            used += int(lens[s])
    return out


def _segment_sums(x64, off_t):
    c = torch.zeros(x64.numel() + 1, dtype=torch.float64, device=x64.device)
    c[1:] = torch.cumsum(x64, 0)
    return (c[off_t[1:]] - c[off_t[:-1]]).cpu().numpy()


def _vocab_rows(V, tokens_np, seed):
    """~64 vocabulary rows: vocabulary-tile edges (256 on the m side of the sweep, 384 on the n side of
    the dW contraction), the ragged last tiles, rows of sampled tokens, random rows."""
    rows = {0, 1, 255, 256, 257, 383, 384, 385, 767, 768, V - 1, V - 2}
    rows.update({V // 256 * 256 - 1, V // 256 * 256, V // 384 * 384 - 1, V // 384 * 384, V // 384 * 384 + 1})
    rows.update(int(t) for t in tokens_np[:: max(1, tokens_np.size // 16)][:16])
    rng = np.random.default_rng(seed)
    while len(rows) < 64:
        rows.add(int(rng.integers(0, V)))
    return np.array(sorted(r for r in rows if 0 <= r < V), dtype=np.int64)


def _oracle_dw_rows(name, b, vsel, coeff, lse_t, slab=32768):
    """Oracle dW[vsel, :] summed over all T token rows, slab by slab (the sum over t is linear)."""
    Wsel = f64(b.W[torch.from_numpy(vsel).to(DEV)])
    tok = b.tokens.cpu().numpy()
    out = np.zeros((vsel.size, b.H.shape[1]))
    t0 = time.time()
    for a in range(0, b.T, slab):
        e = min(b.T, a + slab)
        out += orc.grad_weight_rows(f64(b.H[a:e]), Wsel, vsel, tok[a:e], coeff[a:e], f64(lse_t[a:e]))
        if (a // slab) % 8 == 7 or e == b.T:
            _say(name, f"oracle dW rows: {e}/{b.T} token rows, {time.time() - t0:.0f} s")
    return out


def _slice_batch(b, n_roll=4, cut=256):
    """The first n_roll rollouts of the batch, each cut to `cut` tokens, as one prompt; same W and beta."""
    off = b.seq_offsets.cpu().numpy()
    take = np.minimum(np.diff(off)[:n_roll], cut)
    rows = np.concatenate([np.arange(off[s], off[s] + take[s]) for s in range(n_roll)])
    rt = torch.from_numpy(rows).to(DEV)
    new_off = torch.from_numpy(np.concatenate([[0], np.cumsum(take)]).astype(np.int64)).to(DEV)
    rewards = b.rewards[:n_roll].clone()
    if float(rewards.min()) == float(rewards.max()):
        rewards[0] = 1.0 - rewards[0]          # keep the slice's value estimate non-degenerate
    cfg = synth.reduced(b.cfg, n_prompts=1, n_rollouts=n_roll)
    return synth.RolloutBatch(cfg=cfg, H=b.H[rt].contiguous(), W=b.W, tokens=b.tokens[rt].contiguous(),
                              logq=b.logq[rt].contiguous(), seq_offsets=new_off, rewards=rewards,
                              group_ids=torch.zeros(n_roll, dtype=torch.int32, device=DEV), beta=b.beta)


def _check_grads(got_dH, got_dW, ref):
    gn = rel(grad_norm(got_dH, got_dW), grad_norm(ref["dH"], ref["dW"]))
    assert gn <= 1e-3
    for got, want in ((got_dH, ref["dH"]), (got_dW, ref["dW"])):
        bound = 2e-2 * np.abs(want) + 6e-3 * np.abs(want).max()
        assert np.all(np.abs(got - want) <= bound), float(np.abs(got - want).max())
    return gn


@pytest.mark.parametrize("name", ["qwen1p7b_fwd", "qwen7b", "r1_14b", "long_rollout"])
def test_full_size_configuration(name):
    cfg = synth.CONFIGS[name]
    b = synth.make_batch(cfg, DEV)
    T, d, V = b.T, cfg.d, cfg.V
    off = b.seq_offsets.cpu().numpy()
    lens = np.diff(off)
    gid = b.group_ids.cpu().numpy()
    dt_code = oapl.OAPL_BF16
    # what bench.py does: the default panel, buffers for the longest rollout of the workload
    ws_bytes, panel_rows, panel_bufs = oapl.workspace_bytes_for(T, d, V, b.n_seq, b.n_groups, dt_code, cfg.backward,
                                                                0, int(lens.max()))
    _say(name, f"T={T} d={d} V={V} workspace {ws_bytes / 2**30:.1f} GiB, panels of {panel_rows} rows x {panel_bufs}")
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    res = oapl.loss_fwd_bwd(b.H, b.W, b.tokens, b.logq, b.seq_offsets, b.rewards, b.group_ids, b.n_groups,
                            b.beta, backward=cfg.backward, workspace=ws)
    torch.cuda.synchronize()
    assert oapl.read_device_status(ws) == 0
    assert not oapl.took_two_passes(ws)       # the schedule bench.py times: one sweep over the logits
    W64 = f64(b.W)
    full_oracle = not cfg.backward            # the forward-only configuration: every token row

    # ---- (A) parity with the oracle -----------------------------------------------------------
    rows = np.arange(T) if full_oracle else _sample_rows(off, T, panel_rows, N_SAMPLED, cfg.seed_index)
    rt = torch.from_numpy(rows).to(DEV)
    lp_ref, lse_ref = _oracle_logprobs(name, b, W64, rows, "log-probs")
    lp_err = f64(res.logprob[rt]) - lp_ref
    _say(name, f"log-prob rows={rows.size} max|err|={np.abs(lp_err).max():.3e} mean err={lp_err.mean():+.3e}")
    assert np.abs(lp_err).max() <= 2e-2
    # a systematic per-token error would add up over a rollout: 32768 tokens x 3e-8 = 1e-3
    assert abs(lp_err.mean()) <= 3e-8 + 4 * lp_err.std() / np.sqrt(rows.size)
    assert float(res.logprob.max()) <= 0.0 and bool(torch.isfinite(res.logprob).all())
    # the forward entry point on the same inputs: same log-probs, its log-partition against the oracle's
    lp2, lse2, ws2 = oapl.logprob_fwd(b.H, b.W, b.tokens, want_lse=True)
    torch.cuda.synchronize()
    assert oapl.read_device_status(ws2) == 0
    assert float((lp2 - res.logprob).abs().max()) <= 2e-6
    assert np.abs(f64(lse2[rt]) - lse_ref).max() <= 2e-2
    del lp2, ws2

    vstar_ref = orc.group_value_estimate(f64(b.rewards), gid, b.n_groups, b.beta)
    assert np.abs(f64(res.vstar) - vstar_ref).max() <= 1e-6
    if name == "r1_14b":      # forced all-fail / all-pass prompts: the estimate is the reward itself
        assert res.vstar[0].item() == 0.0 and res.vstar[1].item() == 1.0

    # complete rollouts: Delta_s, delta_s and the loss share, at real rollout lengths
    if full_oracle:
        chosen, lp_full = list(range(b.n_seq)), lp_ref
    else:
        chosen = _complete_rollouts(off, gid, b.n_groups, ROLLOUT_ROW_BUDGET)
    Delta_gpu = f64(res.seq_logratio)
    logq64 = f64(b.logq)
    part_gpu = part_ref = 0.0
    for s in chosen:
        a, e = int(off[s]), int(off[s + 1])
        lp_s = lp_full[a:e] if full_oracle else _oracle_logprobs(name, b, W64, np.arange(a, e), f"rollout {s}")[0]
        D_ref = float(np.sum(lp_s - logq64[a:e]))
        d_ref = b.beta * D_ref - (float(b.rewards[s]) - vstar_ref[gid[s]])
        d_gpu = b.beta * Delta_gpu[s] - (float(b.rewards[s]) - vstar_ref[gid[s]])
        assert abs(Delta_gpu[s] - D_ref) <= 3e-7 * (e - a) + 1e-6 * abs(D_ref) + 1e-6, (s, Delta_gpu[s], D_ref)
        part_gpu += d_gpu * d_gpu
        part_ref += d_ref * d_ref
    if chosen:
        _say(name, f"complete rollouts checked: {len(chosen)} (lengths {[int(lens[s]) for s in chosen]}), "
                   f"loss share rel err {rel(part_gpu, part_ref):.3e}")
        assert rel(part_gpu, part_ref) <= 1e-3
    if full_oracle:           # the whole loss from the oracle's own log-probs
        loss_ref = orc.oapl_loss(orc.sequence_logratio(lp_ref, logq64, off), f64(b.rewards), gid, b.n_groups,
                                 b.beta)[0]
        _say(name, f"full-oracle loss rel err {rel(float(res.loss.item()), loss_ref):.3e}")
        assert rel(float(res.loss.item()), loss_ref) <= 1e-3

    if name == "qwen1p7b_fwd":     # the forward-only configuration also exercises the entropy output at full size
        sub = rows[:: max(1, rows.size // 512)]
        st = torch.from_numpy(sub).to(DEV)
        lp3, ent, ws3 = oapl.logprob_fwd(b.H, b.W, b.tokens, want_entropy=True)
        torch.cuda.synchronize()
        assert oapl.read_device_status(ws3) == 0 and torch.equal(lp3, res.logprob)   # forward-only: same kernels
        ent_ref = orc.token_entropy(f64(b.H[st]), W64)
        _say(name, f"entropy rows={sub.size} max|err|={np.abs(f64(ent[st]) - ent_ref).max():.3e}")
        assert np.abs(f64(ent[st]) - ent_ref).max() <= 2e-2
        assert float(ent.min()) >= 0.0 and float(ent.max()) <= np.log(V) + 1e-4
        del lp3, ent, ws3
        # ... and the sampling kernel at the configuration's own temperature (tokens ~ softmax(z / 0.8))
        from tests.test_gpu_parity import _check_samples
        tok, sc, ws4 = oapl.sample_tokens(b.H, b.W, cfg.token_temp, 2026, want_scores=True)
        torch.cuda.synchronize()
        assert oapl.read_device_status(ws4) == 0
        n_diff = _check_samples(b.H, b.W, cfg.token_temp, 2026, tok, sc, rows=sub)
        _say(name, f"sampled draws checked={sub.size} near-tie differences={n_diff}")
        del tok, sc, ws4

    # ---- (C) properties at full size ----------------------------------------------------------
    seg = _segment_sums(res.logprob.double() - b.logq.double(), b.seq_offsets)
    assert np.all(np.abs(Delta_gpu - seg) <= 3e-7 * np.maximum(lens, 1) + 1e-6 * np.abs(seg) + 1e-6)
    delta = b.beta * Delta_gpu - (f64(b.rewards) - vstar_ref[gid])
    assert rel(float(res.loss.item()), float(np.sum(delta * delta))) <= 1e-5
    if cfg.backward:
        coeff = np.repeat(2.0 * b.beta * delta, lens)          # c_t of every token row
        sub = rows[:: max(1, rows.size // 512)]                # dH rows: a tenth of the sampled token rows
        st = torch.from_numpy(sub).to(DEV)
        g_ref = orc.grad_hidden_rows(f64(b.H[st]), W64, b.tokens[st].cpu().numpy(), coeff[sub], np.arange(sub.size))
        g_gpu = f64(res.dH[st])
        bound = 2e-2 * np.abs(g_ref) + 6e-3 * np.abs(g_ref).max(axis=1, keepdims=True)
        assert np.all(np.abs(g_gpu - g_ref) <= bound), float(np.abs(g_gpu - g_ref).max())
        _say(name, f"dH rows checked={sub.size}")
        # dW rows over ALL token rows (every panel contributes to every row)
        vsel = _vocab_rows(V, b.tokens.cpu().numpy(), cfg.seed_index)
        w_ref = _oracle_dw_rows(name, b, vsel, coeff, lse2)
        w_gpu = f64(res.dW[torch.from_numpy(vsel).to(DEV)])
        w_err = np.abs(w_gpu - w_ref)
        bound = 2e-2 * np.abs(w_ref) + 6e-3 * np.abs(w_ref).max(axis=1, keepdims=True)
        _say(name, f"dW rows checked={vsel.size} max|err|/max|ref|={w_err.max() / np.abs(w_ref).max():.3e} "
                   f"row-norm rel err max={np.max(np.abs(np.linalg.norm(w_gpu, axis=1) / np.linalg.norm(w_ref, axis=1) - 1)):.3e}")
        assert np.all(w_err <= bound), float(w_err.max())
        # The row of a token that was sampled once or twice is essentially c_t (1 - p_y) H_t of that one
        # token.  The soft-max panel holds that entry in bf16 (up to 2^-8 off), and the row factor is
        # corrected for exactly that rounding, so the row's norm must agree far better than 2^-8 = 3.9e-3;
        # what remains is the error of c_t itself (the residual of a rollout of up to 32768 tokens).
        assert np.all(np.abs(np.linalg.norm(w_gpu, axis=1) / np.linalg.norm(w_ref, axis=1) - 1) <= 2e-3)

        assert bool(torch.isfinite(res.dW).all()) and bool(torch.isfinite(res.dH.float()).all())
        col = res.dW.double().sum(0)
        colabs = res.dW.double().abs().sum(0)
        assert float((col.abs() / colabs).max()) <= 5e-3
        # <dH, H> = <dW, W> = sum_t c_t (z_{t,y_t} - E_p z_t).  Rollouts pull in both directions
        # (c_t changes sign with the residual), so the bound is relative to the gross per-token sum.
        per_token = (res.dH.double() * b.H.double()).sum(1)
        a, gross = float(per_token.sum()), float(per_token.abs().sum())
        c = float((res.dW.double() * b.W.double()).sum())
        _say(name, f"<dH,H>={a:.6e} <dW,W>={c:.6e} gross={gross:.3e}")
        assert abs(a - c) <= 2e-3 * gross
    del res, ws, lse2
    torch.cuda.empty_cache()

    # ---- (B) full parity on a slice of the same configuration ---------------------------------
    sb = _slice_batch(b)
    sargs = (sb.H, sb.W, sb.tokens, sb.logq, sb.seq_offsets, sb.rewards, sb.group_ids, 1)
    oargs = (f64(sb.H), W64, sb.tokens.cpu().numpy(), f64(sb.logq), sb.seq_offsets.cpu().numpy(), f64(sb.rewards),
             np.zeros(4, dtype=np.int64), 1)
    sres = oapl.loss_fwd_bwd(*sargs, sb.beta, backward=cfg.backward)
    torch.cuda.synchronize()
    assert oapl.read_device_status(sres.workspace) == 0
    ref = orc.oapl_forward_backward(*oargs, sb.beta, backward=cfg.backward)
    assert np.abs(f64(sres.logprob) - ref["logprob"]).max() <= 2e-2
    assert rel(float(sres.loss.item()), ref["loss"]) <= 1e-3
    _say(name, f"slice T={sb.T} loss_rel={rel(float(sres.loss.item()), ref['loss']):.3e}")
    if not cfg.backward:
        return
    gn = _check_grads(f64(sres.dH), f64(sres.dW), ref)
    _say(name, f"slice gradnorm_rel={gn:.3e}")
    if name != "qwen7b":
        return
    # the experimental section's two constants (beta_1 = 1 in Eq. 2, beta_2 = 1e-3 in Eq. 3) at the real d and V
    b1, b2 = 1.0, float(np.float32(1e-3))
    tres = oapl.loss_fwd_bwd(*sargs, b2, beta_value=b1)
    torch.cuda.synchronize()
    tref = orc.oapl_forward_backward(*oargs, b2, beta_value=b1)
    assert oapl.read_device_status(tres.workspace) == 0 and not oapl.took_two_passes(tres.workspace)
    assert np.abs(f64(tres.vstar) - tref["vstar"]).max() <= 1e-6
    assert rel(float(tres.loss.item()), tref["loss"]) <= 1e-3
    gn = _check_grads(f64(tres.dH), f64(tres.dW), tref)
    _say(name, f"two-beta slice loss_rel={rel(float(tres.loss.item()), tref['loss']):.3e} gradnorm_rel={gn:.3e}")
    # the GRPO baseline at the real d and V (ratios well inside one branch of the clip, both branches present)
    from tests.test_gpu_parity import _grpo_check, _grpo_inputs
    logq, logp_old = _grpo_inputs(sb, 77)
    gres = oapl.grpo_loss_fwd_bwd(sb.H, sb.W, sb.tokens, logq, logp_old, sb.seq_offsets, sb.rewards, sb.group_ids, 1)
    torch.cuda.synchronize()
    assert not oapl.took_two_passes(gres.workspace)
    gref = _grpo_check(sb, logq, logp_old, gres, lp_tol=2e-2, rel_tol=1e-3, g_rtol=2e-2, g_atol_frac=6e-3)
    gn = rel(grad_norm(f64(gres.dH), f64(gres.dW)), grad_norm(gref["dH"], gref["dW"]))
    _say(name, f"GRPO slice gradnorm_rel={gn:.3e}")
