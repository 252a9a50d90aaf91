"""The seeded input generator: shapes, determinism and the stated distributions."""
import numpy as np
import torch

from workloads import synth


def test_tiny_config_shapes_and_determinism():
    cfg = synth.CONFIGS["tiny_f32"]
    a = synth.make_batch(cfg, "cpu")
    b = synth.make_batch(cfg, "cpu")
    assert a.T == 256 and a.H.shape == (256, 64) and a.W.shape == (1024, 64)
    assert a.H.dtype == torch.float32 and a.tokens.dtype == torch.int32
    assert a.seq_offsets.tolist() == list(range(0, 257, 32))
    assert a.group_ids.tolist() == [0, 0, 0, 0, 1, 1, 1, 1]
    assert set(a.rewards.tolist()) <= {0.0, 1.0}
    for x, y in ((a.H, b.H), (a.W, b.W), (a.tokens, b.tokens), (a.logq, b.logq), (a.rewards, b.rewards)):
        assert torch.equal(x, y)
    assert int(a.tokens.min()) >= 0 and int(a.tokens.max()) < 1024
    assert abs(float(a.H.std()) - 1.0) < 0.02
    assert abs(float(a.W.std()) - 0.125) < 0.005
    # inference log-probs are log-probs plus a little noise: close to -ln V - 1/2
    assert abs(float(a.logq.mean()) + np.log(1024) + 0.5) < 0.2


def test_lognormal_lengths_are_truncated_and_packed():
    cfg = synth.reduced(synth.CONFIGS["qwen7b"], d=64, V=512, len_median=40, len_max=80, len_min=4)
    b = synth.make_batch(cfg, "cpu")
    lens = np.diff(b.seq_offsets.numpy())
    assert lens.min() >= 4 and lens.max() <= 80 and (lens == 80).any()
    assert b.T == int(lens.sum()) and b.H.dtype == torch.bfloat16
    assert b.n_seq == 64 and b.n_groups == 8


def test_forced_degenerate_groups_in_beta_prompt_rewards():
    cfg = synth.reduced(synth.CONFIGS["r1_14b"], d=64, V=256, len_median=8, len_max=16, len_min=2)
    b = synth.make_batch(cfg, "cpu")
    r = b.rewards.numpy().reshape(8, 16)
    assert (r[0] == 0).all() and (r[1] == 1).all()


def test_policy_tokens_prefer_likely_tokens_and_lagged_weights_shift_logq():
    cfg = synth.reduced(synth.CONFIGS["qwen1p7b_fwd"], d=64, V=300, n_prompts=2, n_rollouts=2, len_fixed=64)
    b = synth.make_batch(cfg, "cpu")
    base = synth.engine_logprobs(b.H, b.W, b.tokens)
    # tokens sampled from the policy are (on average) more likely than uniform ones
    assert float(base.mean()) > -np.log(300) - 0.5 + 0.3
    cfg5 = synth.reduced(synth.CONFIGS["long_rollout"], d=64, V=300, n_prompts=2, n_rollouts=2, len_fixed=64)
    b5 = synth.make_batch(cfg5, "cpu")
    base5 = synth.engine_logprobs(b5.H, b5.W, b5.tokens)
    diff = (b5.logq - base5).abs()
    assert 1e-3 < float(diff.mean()) < 1.0
