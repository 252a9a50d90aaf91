"""The C-ABI library: it loads, exports every declared symbol, and its host-side
argument checks answer without a GPU (they return before any launch)."""
import ctypes
import os
import re

import pytest

from paper_2602_19362_amd import oapl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "oapl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(oapl_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert "oapl_logprob_fwd" in names and "oapl_loss_fwd_bwd" in names
    handle = ctypes.CDLL(oapl.lib_path())
    for n in names:
        assert hasattr(handle, n), n
    assert set(names) == set(oapl._SIGNATURES), "binding and header disagree"


def test_status_strings():
    L = oapl.lib()
    assert L.oapl_status_string(0) == b"ok"
    seen = {L.oapl_status_string(i) for i in range(11)}
    assert len(seen) == 11 and L.oapl_status_string(77) == b"unknown status"


def test_workspace_bytes_host_logic():
    wb = oapl.workspace_bytes
    small = wb(256, 64, 1024, 8, 2, oapl.OAPL_F32, False)
    assert small > 0 and small % 256 == 0
    assert wb(256, 64, 1024, 8, 2, oapl.OAPL_F32, True) > small
    # the bf16 backward workspace holds one pair of soft-max panels (tokens x V and V x tokens) when
    # T fits one panel (at most 12288 rows by default) and two pairs beyond that; they stop growing at
    # the panel size, after which only the per-token buffers and the packed copy of H grow with T
    panel = 12288 * 151936 * 2
    a = wb(12288, 4096, 151936, 64, 8, oapl.OAPL_BF16, True)
    b = wb(1 << 20, 4096, 151936, 64, 8, oapl.OAPL_BF16, True)
    c = wb(1 << 21, 4096, 151936, 64, 8, oapl.OAPL_BF16, True)
    per_token = 2 * 4096 + 2048                       # packed H row + per-token scalars and soft-max partials
    assert 2 * panel < a < 3 * panel
    assert 2 * panel < b - a < 2 * panel + (1 << 20) * per_token
    assert c - b < (1 << 20) * per_token
    # invalid sizes
    assert wb(-1, 64, 1024, 8, 2, 0, False) == 0
    assert wb(256, 0, 1024, 8, 2, 0, False) == 0
    assert wb(256, 64, 0, 8, 2, 0, False) == 0
    assert wb(256, 64, 1024, 8, 0, 0, False) == 0
    assert wb(256, 64, 1024, 8, 2, 5, False) == 0
    assert wb(256, 64, (1 << 21) + 1, 8, 2, 0, False) == 0 and wb(256, (1 << 21) + 8, 1024, 8, 2, 0, False) == 0
    assert wb(65535 * 256 + 1, 64, 1024, 8, 2, oapl.OAPL_BF16, False) == 0
    assert wb(256, 60, 1024, 8, 2, oapl.OAPL_BF16, False) == 0     # bf16 rows must be 16-byte multiples
    assert wb(65535 * 64 + 1, 64, 1024, 8, 2, oapl.OAPL_F32, False) == 0    # fp32 token tiles index gridDim.y
    assert wb(65535 * 64, 64, 1024, 8, 2, oapl.OAPL_F32, False) > 0
    assert wb(256, 64, 1024, 1 << 20, 1 << 13, 0, False) == 0      # n_seq * n_groups above 2^32
    assert wb(256, 64, 1024, 1 << 20, 1 << 12, 0, False) > 0
    assert wb(0, 64, 1024, 0, 1, oapl.OAPL_BF16, True) > 0          # an empty batch is legal


def test_workspace_is_the_memory_budget():
    """oapl_workspace_bytes_for: panel size and panel buffers set the workspace; the plan reports both."""
    wbf = oapl.workspace_bytes_for
    args = (140897, 4096, 151936, 64, 8, oapl.OAPL_BF16, True)
    full = oapl.workspace_bytes(*args)
    assert wbf(*args, 0, 0) == (full, 12288, 2)                    # default: 32 token tiles, two buffers
    per_row = 151936 * 2 * 2                                        # both packed copies, bf16
    prev = None
    for cap in (384, 1000, 6144, 12288, 24576, 1 << 40):
        nbytes, rows, bufs = wbf(*args, cap, 0)
        assert nbytes > 0 and rows % 384 == 0 and 384 <= rows <= max(min(cap, 12288), 384) and bufs == 2
        assert 2 * rows * per_row < nbytes < 2 * rows * per_row * 1.02 + (5 << 30)
        assert prev is None or nbytes >= prev
        prev = nbytes
    assert full < 18 << 30
    # buffers for longer rollouts: 1 + ceil(len / panel rows), never more than the batch has panels
    assert wbf(*args, 0, 12288)[2] == 2 and wbf(*args, 0, 12289)[2] == 3 and wbf(*args, 0, 32768)[2] == 4
    assert wbf(*args, 0, 10 ** 9)[2] == 12                          # ceil(140897 / 12288) panels in all
    a3, _, _ = wbf(*args, 0, 12289)
    assert 0.98 * 12288 * per_row < a3 - full < 1.02 * 12288 * per_row
    assert wbf(*args, 6144, 32768)[1:] == (6144, 2)                 # smaller panels: always two buffers
    # one panel is enough when the batch fits it
    assert wbf(6000, 4096, 151936, 8, 1, oapl.OAPL_BF16, True, 0, 50000)[1:] == (6144, 1)
    # d = 5120: 20 row tiles of dH per token tile; the plan picks a panel that fills whole rounds of 256 workgroups
    rows = wbf(896842, 5120, 151936, 128, 8, oapl.OAPL_BF16, True, 0, 0)[1]
    assert rows % 384 == 0 and 6144 <= rows <= 12288 and (20 * rows // 384) % 256 in (0, *range(240, 256))
    # fp32: the panel is the logit-gradient block [rows, V]
    a, ra, _ = wbf(5000, 64, 1024, 8, 2, oapl.OAPL_F32, True, 0, 0)
    b, rb, _ = wbf(5000, 64, 1024, 8, 2, oapl.OAPL_F32, True, 512, 0)
    assert (ra, rb) == (4096, 512) and a - b == (4096 - 512) * 1024 * 4
    # invalid sizes answer 0 like oapl_workspace_bytes
    assert wbf(-1, 64, 1024, 8, 2, 0, True, 512, 0) == (0, 0, 0)


def test_host_side_errors_return_before_any_launch():
    L = oapl.lib()
    one = ctypes.c_void_p(256)          # never dereferenced: the checks below fail first
    # dtype / shape / null
    assert L.oapl_logprob_fwd(one, one, one, 4, 8, 8, 7, one, None, None, one, 1 << 20, None) == 3
    assert L.oapl_logprob_fwd(one, one, one, 4, 0, 8, 0, one, None, None, one, 1 << 20, None) == 2
    assert L.oapl_logprob_fwd(None, one, one, 4, 8, 8, 0, one, None, None, one, 1 << 20, None) == 1
    # workspace: null, misaligned, too small
    assert L.oapl_logprob_fwd(one, one, one, 4, 8, 8, 0, one, None, None, None, 1 << 20, None) == 7
    assert L.oapl_logprob_fwd(one, one, one, 4, 8, 8, 0, one, None, None, ctypes.c_void_p(260), 1 << 20, None) == 7
    assert L.oapl_logprob_fwd(one, one, one, 4, 8, 8, 0, one, None, None, one, 16, None) == 7

    def loss(beta=1.0, scale=1.0, dH=one, dW=one, dtype=0, n_groups=1, ws_bytes=1 << 24):
        return L.oapl_loss_fwd_bwd(one, one, one, one, one, one, one, 4, 8, 8, 2, n_groups, dtype,
                                   beta, scale, one, None, None, None, dH, dW, one, ws_bytes, None)
    assert loss(beta=0.0) == 6 and loss(beta=-1.0) == 6 and loss(beta=float("nan")) == 6
    assert loss(beta=float("inf")) == 6 and loss(scale=float("inf")) == 6
    assert loss(dH=None) == 1 and loss(dW=None) == 1          # gradients come as a pair
    assert loss(dtype=9) == 3 and loss(n_groups=0) == 2 and loss(ws_bytes=64) == 7
    def two_beta(beta_loss=1.0, flags=0):
        return L.oapl_loss_fwd_bwd_two_beta(one, one, one, one, one, one, one, 4, 8, 8, 2, 1, 0, 1.0, beta_loss, 1.0,
                                            flags, one, None, None, None, one, one, one, 1 << 24, None)
    assert two_beta(beta_loss=0.0) == 6
    assert two_beta(flags=2) == 2 and two_beta(flags=0x80000000) == 2       # unknown option bits
    # the entry point that allocates nothing: same checks, and sizes beyond its 64 MiB scratch are refused
    def noalloc(beta=1.0, T=4, d=8, V=8, dtype=0, dW=one):
        return L.oapl_loss_fwd_bwd_noalloc(one, one, one, one, one, one, one, T, d, V, 2, 1, dtype, beta, 1.0,
                                           one, None, None, None, one, dW, None)
    assert noalloc(beta=0.0) == 6 and noalloc(dtype=4) == 3 and noalloc(d=0) == 2 and noalloc(dW=None) == 1
    assert noalloc(T=1000, d=4096, V=151936, dtype=1) == 10
    assert L.oapl_status_string(10).startswith(b"sizes need more than")
    # GRPO baseline: clip in [0, 1), adv_eps >= 0, finite scale; gradients as a pair; logp_old required
    def grpo(clip=0.2, eps=1e-6, scale=1.0, old=one, dH=one, dW=one, dtype=0, flags=0):
        return L.oapl_grpo_loss_fwd_bwd(one, one, one, one, old, one, one, one, 4, 8, 8, 2, 1, dtype, clip, eps,
                                        scale, flags, one, None, None, dH, dW, one, 1 << 24, None)
    assert grpo(clip=1.0) == 6 and grpo(clip=-0.1) == 6 and grpo(clip=float("nan")) == 6
    assert grpo(eps=-1.0) == 6 and grpo(eps=float("inf")) == 6 and grpo(scale=float("nan")) == 6
    assert grpo(old=None) == 1 and grpo(dH=None) == 1 and grpo(dtype=5) == 3 and grpo(flags=4) == 2
    # sampling: temperature must be positive and finite
    assert L.oapl_sample_tokens(one, one, 4, 8, 8, 0, 0.0, 1, one, None, one, 1 << 20, None) == 6
    assert L.oapl_sample_tokens(one, one, 4, 8, 8, 0, float("nan"), 1, one, None, one, 1 << 20, None) == 6
    assert L.oapl_sample_tokens(one, one, 4, 8, 8, 0, 1.0, 1, None, None, one, 1 << 20, None) == 1
    assert L.oapl_sample_tokens(one, one, 4, 8, 8, 3, 1.0, 1, one, None, one, 1 << 20, None) == 3
    assert L.oapl_segmented_sum_f32(None, one, 3, one, None) == 1
    assert L.oapl_segmented_sum_f32(one, one, -1, one, None) == 2
    assert L.oapl_segmented_sum_f32(None, None, 0, None, None) == 0
    assert L.oapl_read_device_status(None, None, None) == 1


def test_product_path_has_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("checked on the CPU-only box")
    H = torch.zeros(4, 8)
    W = torch.zeros(8, 8)
    tok = torch.zeros(4, dtype=torch.int32)
    with pytest.raises(ValueError):
        oapl.logprob_fwd(H, W, tok)       # host tensors are refused, nothing is computed on the CPU


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr + r.stdout
