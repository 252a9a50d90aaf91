"""Helpers shared by the GPU parity tests (no arithmetic of the method here)."""
import numpy as np
import torch

from oracle import oapl_oracle as orc


def f64(t):
    """Exact widening of a tensor (bf16 / fp32 / ints) to a float64 numpy array."""
    return t.detach().cpu().to(torch.float64).numpy()


def oracle_full(b, beta=None, beta_value=None, loss_scale=1.0, backward=True):
    """The CPU oracle on exactly the tensors the GPU path gets."""
    return orc.oapl_forward_backward(
        f64(b.H), f64(b.W), b.tokens.cpu().numpy(), f64(b.logq), b.seq_offsets.cpu().numpy(),
        f64(b.rewards), b.group_ids.cpu().numpy(), b.n_groups, b.beta if beta is None else beta,
        beta_value=beta_value, loss_scale=loss_scale, backward=backward)


def rel(a, b):
    return abs(a - b) / max(abs(b), 1e-300)


def grad_norm(*arrays):
    return float(np.sqrt(sum(float((np.asarray(a, dtype=np.float64) ** 2).sum()) for a in arrays)))
