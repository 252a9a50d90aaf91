"""Guard bands: every output and the workspace of the entry points live inside larger buffers
filled with a canary pattern; after the call the bands on both sides must be untouched.  An
out-of-tile write at a ragged edge that lands in another live allocation would pass every parity
test; here it lands in a band."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_19362_amd import oapl
from workloads import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CANARY = 0xA5


class Banded:
    """A device buffer of `nbytes` with `band` canary bytes before and after it."""

    def __init__(self, nbytes, band):
        assert band % 256 == 0
        self.band, self.nbytes = band, nbytes
        self.raw = torch.full((nbytes + 2 * band,), CANARY, dtype=torch.uint8, device=DEV)
        assert self.raw.data_ptr() % 256 == 0

    @property
    def ptr(self):
        return self.raw.data_ptr() + self.band

    def view(self, dtype, shape):
        return self.raw[self.band:self.band + self.nbytes].view(dtype).view(shape)

    def intact(self):
        lo = self.raw[:self.band]
        hi = self.raw[self.band + self.nbytes:]
        return bool((lo == CANARY).all()) and bool((hi == CANARY).all())


def _loss_call(b, n_groups, beta, flags, ws_bytes, big_band):
    """oapl_loss_fwd_bwd_two_beta through the C ABI with every output and the workspace banded."""
    T, d = b.H.shape
    V = b.W.shape[0]
    n_seq = b.rewards.shape[0]
    esize = b.H.element_size()
    bufs = dict(loss=Banded(4, 4096), logprob=Banded(4 * T, 4096), seq_lr=Banded(4 * n_seq, 4096),
                vstar=Banded(4 * n_groups, 4096), dH=Banded(esize * T * d, big_band), dW=Banded(4 * V * d, big_band),
                ws=Banded(ws_bytes, big_band))
    dt = oapl.OAPL_BF16 if b.H.dtype == torch.bfloat16 else oapl.OAPL_F32
    rc = oapl.lib().oapl_loss_fwd_bwd_two_beta(
        b.H.data_ptr(), b.W.data_ptr(), b.tokens.data_ptr(), b.logq.data_ptr(), b.seq_offsets.data_ptr(),
        b.rewards.data_ptr(), b.group_ids.data_ptr(), T, d, V, n_seq, n_groups, dt, float(beta), float(beta), 1.0,
        flags, bufs["loss"].ptr, bufs["logprob"].ptr, bufs["seq_lr"].ptr, bufs["vstar"].ptr, bufs["dH"].ptr,
        bufs["dW"].ptr, bufs["ws"].ptr, ws_bytes, torch.cuda.current_stream().cuda_stream)
    assert rc == 0, rc
    torch.cuda.synchronize()
    status = ctypes.c_int32(-1)
    assert oapl.lib().oapl_read_device_status(bufs["ws"].ptr, None, ctypes.byref(status)) == 0 and status.value == 0
    for name, buf in bufs.items():
        assert buf.intact(), f"{name}: guard band overwritten"
    # the outputs themselves were written (no canary-valued floats left behind) and are finite
    assert bool(torch.isfinite(bufs["loss"].view(torch.float32, (1,))).all())
    assert bool(torch.isfinite(bufs["logprob"].view(torch.float32, (T,))).all())
    assert bool(torch.isfinite(bufs["dW"].view(torch.float32, (V, d))).all())
    assert bool(torch.isfinite(bufs["dH"].view(b.H.dtype, (T, d)).float()).all())
    return bufs


def _ragged_batch(dtype, d, V, lens, seed):
    from tests.test_gpu_parity import _custom_batch
    return _custom_batch(dtype, d=d, V=V, lens=lens, n_groups=2, seed=seed, beta=0.7, noise=0.1)


@pytest.mark.parametrize("flags", [0, oapl.OAPL_FLAG_TWO_PASS])
@pytest.mark.parametrize("d,V,lens,cap", [
    (320, 1544, [300, 17, 0, 383, 200, 100], 384),       # T = 1000: 3 one-tile panels, ragged last token tile; V = 6*256 + 8; d = 5*64
    (256, 1544, [100, 3, 0, 257, 64, 1, 200, 75], 0),    # one panel of two token tiles
    (64, 264, [511, 2], 0),                               # second vocabulary tile almost empty
])
def test_bf16_ragged_shapes_stay_inside_their_buffers(d, V, lens, cap, flags):
    b = _ragged_batch("bf16", d, V, lens, seed=41)
    ws_bytes, rows, _ = oapl.workspace_bytes_for(b.T, d, V, len(lens), 2, oapl.OAPL_BF16, True, cap, 0)
    assert cap == 0 or (rows == cap and b.T > 2 * cap)
    _loss_call(b, 2, 0.7, flags, ws_bytes, big_band=1 << 20)


def test_f32_ragged_shapes_stay_inside_their_buffers():
    lens = [0, 1, 37, 64, 0, 129, 5, 64]
    b = _ragged_batch("f32", 72, 1000, lens, seed=42)
    ws_bytes, _, _ = oapl.workspace_bytes_for(b.T, 72, 1000, len(lens), 2, oapl.OAPL_F32, True, 100, 0)
    _loss_call(b, 2, 0.7, 0, ws_bytes, big_band=1 << 20)


def test_forward_and_sampling_entry_points_stay_inside_their_buffers():
    b = _ragged_batch("bf16", 320, 1544, [300, 17, 0, 383, 200, 100], seed=43)
    T, d, V = b.T, 320, 1544
    ws_bytes = oapl.workspace_bytes(T, d, V, 0, 1, oapl.OAPL_BF16, False)
    st = torch.cuda.current_stream().cuda_stream
    ws, lp, lse, ent = Banded(ws_bytes, 1 << 20), Banded(4 * T, 4096), Banded(4 * T, 4096), Banded(4 * T, 4096)
    assert oapl.lib().oapl_logprob_fwd(b.H.data_ptr(), b.W.data_ptr(), b.tokens.data_ptr(), T, d, V, oapl.OAPL_BF16,
                                       lp.ptr, lse.ptr, ent.ptr, ws.ptr, ws_bytes, st) == 0
    tok, sc = Banded(4 * T, 4096), Banded(4 * T, 4096)
    ws2 = Banded(ws_bytes, 1 << 20)
    assert oapl.lib().oapl_sample_tokens(b.H.data_ptr(), b.W.data_ptr(), T, d, V, oapl.OAPL_BF16, 0.8, 7, tok.ptr,
                                         sc.ptr, ws2.ptr, ws_bytes, st) == 0
    torch.cuda.synchronize()
    for name, buf in dict(ws=ws, lp=lp, lse=lse, ent=ent, tok=tok, sc=sc, ws2=ws2).items():
        assert buf.intact(), f"{name}: guard band overwritten"
    assert bool(torch.isfinite(lp.view(torch.float32, (T,))).all())
    t = tok.view(torch.int32, (T,))
    assert int(t.min()) >= 0 and int(t.max()) < V


def test_full_size_configuration_stays_inside_its_buffers():
    """The benchmark's workload (d = 4096, V = 151936, T = 140897: 12 panels, ragged last token tile and
    last vocabulary tile) with 16 MiB bands around dH, dW and the workspace."""
    cfg = synth.CONFIGS["qwen7b"]
    b = synth.make_batch(cfg, DEV)
    longest = int((b.seq_offsets[1:] - b.seq_offsets[:-1]).max().item())
    ws_bytes, rows, bufs = oapl.workspace_bytes_for(b.T, cfg.d, cfg.V, b.n_seq, b.n_groups, oapl.OAPL_BF16, True, 0,
                                                    longest)
    print(f"[guard] T={b.T} panels of {rows} x {bufs}, workspace {ws_bytes / 2**30:.1f} GiB", flush=True)
    out = _loss_call(b, b.n_groups, cfg.beta, 0, ws_bytes, big_band=16 << 20)
    two_pass = ctypes.c_int32(-1)
    assert oapl.lib().oapl_read_path_taken(out["ws"].ptr, None, ctypes.byref(two_pass)) == 0 and two_pass.value == 0
