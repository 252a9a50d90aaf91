"""ctypes binding of liboapl_hip.so (the C ABI declared in include/oapl.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory and the current HIP stream.  There is
no fallback: if the shared library has not been built, or no GPU is present,
the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple, Optional

import torch

_LIB_NAME = "liboapl_hip.so"
_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), _LIB_NAME)

OAPL_F32 = 0
OAPL_BF16 = 1
OAPL_FLAG_TWO_PASS = 1

STATUS_NAMES = {
    0: "OAPL_OK", 1: "OAPL_ERR_NULL", 2: "OAPL_ERR_SHAPE", 3: "OAPL_ERR_DTYPE", 4: "OAPL_ERR_OFFSETS",
    5: "OAPL_ERR_GROUP", 6: "OAPL_ERR_BETA", 7: "OAPL_ERR_WORKSPACE", 8: "OAPL_ERR_HIP", 9: "OAPL_ERR_TOKEN_RANGE",
    10: "OAPL_ERR_SCRATCH_LIMIT",
}

# Every symbol include/oapl.h declares, with its ctypes signature.
_c = ctypes
_SIGNATURES = {
    "oapl_status_string": (_c.c_char_p, [_c.c_int32]),
    "oapl_workspace_bytes": (_c.c_size_t, [_c.c_int64, _c.c_int32, _c.c_int32, _c.c_int32, _c.c_int32, _c.c_int32,
                                           _c.c_int32]),
    "oapl_workspace_bytes_for": (_c.c_size_t, [_c.c_int64, _c.c_int32, _c.c_int32, _c.c_int32, _c.c_int32,
                                               _c.c_int32, _c.c_int32, _c.c_int64, _c.c_int64,
                                               _c.POINTER(_c.c_int64), _c.POINTER(_c.c_int32)]),
    "oapl_logprob_fwd": (_c.c_int32, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int32, _c.c_int32,
                                      _c.c_int32, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_size_t,
                                      _c.c_void_p]),
    "oapl_sample_tokens": (_c.c_int32, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int32, _c.c_int32, _c.c_int32,
                                        _c.c_float, _c.c_uint64, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_size_t,
                                        _c.c_void_p]),
    "oapl_loss_fwd_bwd": (_c.c_int32, [_c.c_void_p] * 7 + [_c.c_int64] + [_c.c_int32] * 5 + [_c.c_float] * 2 +
                          [_c.c_void_p] * 7 + [_c.c_size_t, _c.c_void_p]),
    "oapl_loss_fwd_bwd_two_beta": (_c.c_int32, [_c.c_void_p] * 7 + [_c.c_int64] + [_c.c_int32] * 5 + [_c.c_float] * 3 +
                                   [_c.c_uint32] + [_c.c_void_p] * 7 + [_c.c_size_t, _c.c_void_p]),
    "oapl_loss_fwd_bwd_noalloc": (_c.c_int32, [_c.c_void_p] * 7 + [_c.c_int64] + [_c.c_int32] * 5 + [_c.c_float] * 2 +
                                  [_c.c_void_p] * 7),
    "oapl_grpo_loss_fwd_bwd": (_c.c_int32, [_c.c_void_p] * 8 + [_c.c_int64] + [_c.c_int32] * 5 + [_c.c_float] * 3 +
                               [_c.c_uint32] + [_c.c_void_p] * 6 + [_c.c_size_t, _c.c_void_p]),
    "oapl_segmented_sum_f32": (_c.c_int32, [_c.c_void_p, _c.c_void_p, _c.c_int32, _c.c_void_p, _c.c_void_p]),
    "oapl_read_device_status": (_c.c_int32, [_c.c_void_p, _c.c_void_p, _c.POINTER(_c.c_int32)]),
    "oapl_read_path_taken": (_c.c_int32, [_c.c_void_p, _c.c_void_p, _c.POINTER(_c.c_int32)]),
    "oapl_timing_enable": (_c.c_int32, [_c.c_int32]),
    "oapl_timing_read": (_c.c_int32, [_c.c_int32, _c.POINTER(_c.c_double), _c.POINTER(_c.c_int64)]),
}

DENSE_KERNELS = ("k_fwd_lse", "k_bwd_dz", "k_bwd_dh", "k_bwd_dw", "k_fwd_sample", "k_sweep")

_lib = None


class OaplError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = STATUS_NAMES.get(status, str(status))
        try:
            msg += ": " + lib().oapl_status_string(status).decode()
        except Exception:
            pass
        super().__init__(f"{where} failed with {msg}")


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """Loads the shared library once; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
                "There is no CPU fallback.")
        handle = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return OAPL_F32
    if t.dtype == torch.bfloat16:
        return OAPL_BF16
    raise TypeError(f"H and W must be float32 or bfloat16, got {t.dtype}")


def _dev(t: Optional[torch.Tensor], dtype: torch.dtype, name: str, device) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.device != device:
        raise ValueError(f"{name} must live on {device}")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def workspace_bytes(T: int, d: int, V: int, n_seq: int, n_groups: int, dtype: int, with_backward: bool,
                    max_panel_rows: Optional[int] = None, max_rollout_len: Optional[int] = None) -> int:
    """oapl_workspace_bytes, or oapl_workspace_bytes_for when a panel cap or a rollout length is given."""
    if max_panel_rows is None and max_rollout_len is None:
        return int(lib().oapl_workspace_bytes(T, d, V, n_seq, n_groups, dtype, 1 if with_backward else 0))
    return workspace_bytes_for(T, d, V, n_seq, n_groups, dtype, with_backward, max_panel_rows or 0,
                               max_rollout_len or 0)[0]


def workspace_bytes_for(T: int, d: int, V: int, n_seq: int, n_groups: int, dtype: int, with_backward: bool,
                        max_panel_rows: int = 0, max_rollout_len: int = 0):
    """oapl_workspace_bytes_for: (bytes, panel rows, panel buffers) of the plan."""
    rows = ctypes.c_int64(0)
    bufs = ctypes.c_int32(0)
    n = lib().oapl_workspace_bytes_for(T, d, V, n_seq, n_groups, dtype, 1 if with_backward else 0,
                                       int(max_panel_rows), int(max_rollout_len), ctypes.byref(rows),
                                       ctypes.byref(bufs))
    return int(n), int(rows.value), int(bufs.value)


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> torch.Tensor:
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    if workspace.dtype != torch.uint8 or not workspace.is_contiguous() or workspace.device != device:
        raise ValueError("workspace must be a contiguous uint8 tensor on the inputs' device")
    return workspace


def read_device_status(workspace: torch.Tensor) -> int:
    out = ctypes.c_int32(0)
    rc = lib().oapl_read_device_status(workspace.data_ptr(), _stream(workspace.device), ctypes.byref(out))
    if rc != 0:
        raise OaplError(rc, "oapl_read_device_status")
    return int(out.value)


def took_two_passes(workspace: torch.Tensor) -> bool:
    """oapl_read_path_taken: True if the last loss call on this workspace fell back to the two-pass schedule."""
    out = ctypes.c_int32(0)
    rc = lib().oapl_read_path_taken(workspace.data_ptr(), _stream(workspace.device), ctypes.byref(out))
    if rc != 0:
        raise OaplError(rc, "oapl_read_path_taken")
    return bool(out.value)


def _check_device(t: torch.Tensor) -> None:
    """The C ABI works on the current HIP device: the inputs must live there."""
    if not t.is_cuda:
        raise ValueError("inputs must be device tensors (there is no CPU path)")
    if t.device.index != torch.cuda.current_device():
        raise ValueError(f"inputs live on {t.device} but the current device is cuda:{torch.cuda.current_device()}; "
                         "wrap the call in torch.cuda.device(...)")


def logprob_fwd(H: torch.Tensor, W: torch.Tensor, tokens: torch.Tensor, *, want_lse: bool = False,
                want_entropy: bool = False, workspace: Optional[torch.Tensor] = None):
    """oapl_logprob_fwd: per-token log-probs of the sampled tokens (and lse, and the policy entropy).

    Returns (logprob, [lse], [entropy], workspace) with the optional items present when asked for.
    """
    L = lib()
    _check_device(H)
    dt = _dtype_code(H)
    T, d = H.shape
    V = W.shape[0]
    if W.shape[1] != d or tokens.shape != (T,):
        raise ValueError("shape mismatch between H, W and tokens")
    dev = H.device
    nbytes = workspace_bytes(T, d, V, 0, 1, dt, False)
    if nbytes == 0:
        raise OaplError(2, "oapl_workspace_bytes")
    ws = _workspace(nbytes, dev, workspace)
    logprob = torch.empty(T, dtype=torch.float32, device=dev)
    lse = torch.empty(T, dtype=torch.float32, device=dev) if want_lse else None
    ent = torch.empty(T, dtype=torch.float32, device=dev) if want_entropy else None
    rc = L.oapl_logprob_fwd(_dev(H, H.dtype, "H", dev), _dev(W, H.dtype, "W", dev),
                            _dev(tokens, torch.int32, "tokens", dev), T, d, V, dt, logprob.data_ptr(),
                            lse.data_ptr() if want_lse else None, ent.data_ptr() if want_entropy else None,
                            ws.data_ptr(), ws.numel(), _stream(dev))
    if rc != 0:
        raise OaplError(rc, "oapl_logprob_fwd")
    return tuple(x for x in (logprob, lse, ent) if x is not None) + (ws,)


def sample_tokens(H: torch.Tensor, W: torch.Tensor, temperature: float, seed: int, *, want_scores: bool = False,
                  workspace: Optional[torch.Tensor] = None):
    """oapl_sample_tokens: one Gumbel-max draw per row from softmax(H W^T / temperature)."""
    _check_device(H)
    dt = _dtype_code(H)
    T, d = H.shape
    V = W.shape[0]
    if W.shape[1] != d:
        raise ValueError("shape mismatch between H and W")
    dev = H.device
    nbytes = workspace_bytes(T, d, V, 0, 1, dt, False)
    if nbytes == 0:
        raise OaplError(2, "oapl_workspace_bytes")
    ws = _workspace(nbytes, dev, workspace)
    tokens = torch.empty(T, dtype=torch.int32, device=dev)
    scores = torch.empty(T, dtype=torch.float32, device=dev) if want_scores else None
    rc = lib().oapl_sample_tokens(_dev(H, H.dtype, "H", dev), _dev(W, H.dtype, "W", dev), T, d, V, dt,
                                  float(temperature), int(seed) & 0xFFFFFFFFFFFFFFFF, tokens.data_ptr(),
                                  scores.data_ptr() if want_scores else None, ws.data_ptr(), ws.numel(), _stream(dev))
    if rc != 0:
        raise OaplError(rc, "oapl_sample_tokens")
    return (tokens, scores, ws) if want_scores else (tokens, ws)


class LossResult(NamedTuple):
    loss: torch.Tensor            # [1] float32
    logprob: torch.Tensor         # [T] float32
    seq_logratio: torch.Tensor    # [N] float32
    vstar: torch.Tensor           # [P] float32
    dH: Optional[torch.Tensor]    # [T, d] in H's dtype
    dW: Optional[torch.Tensor]    # [V, d] float32
    workspace: torch.Tensor


def loss_fwd_bwd(H, W, tokens, logq, seq_offsets, rewards, group_ids, n_groups: int, beta: float, *,
                 beta_value: Optional[float] = None, loss_scale: float = 1.0, backward: bool = True,
                 two_pass: bool = False, max_panel_rows: Optional[int] = None,
                 max_rollout_len: Optional[int] = None, workspace: Optional[torch.Tensor] = None,
                 dH: Optional[torch.Tensor] = None, dW: Optional[torch.Tensor] = None) -> LossResult:
    """oapl_loss_fwd_bwd (or the two-beta entry point when beta_value or two_pass is given).

    max_panel_rows / max_rollout_len only size the workspace this wrapper allocates when none is
    passed; the library derives its plan from the bytes it is handed.
    """
    L = lib()
    _check_device(H)
    dt = _dtype_code(H)
    T, d = H.shape
    V = W.shape[0]
    n_seq = rewards.shape[0]
    if W.shape[1] != d or tokens.shape != (T,) or logq.shape != (T,) or seq_offsets.shape != (n_seq + 1,) \
            or group_ids.shape != (n_seq,):
        raise ValueError("shape mismatch between the inputs")
    dev = H.device
    nbytes = workspace_bytes(T, d, V, n_seq, n_groups, dt, backward, max_panel_rows, max_rollout_len)
    if nbytes == 0:
        raise OaplError(2, "oapl_workspace_bytes")
    ws = _workspace(nbytes, dev, workspace)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    logprob = torch.empty(T, dtype=torch.float32, device=dev)
    seq_lr = torch.empty(n_seq, dtype=torch.float32, device=dev)
    vstar = torch.empty(n_groups, dtype=torch.float32, device=dev)
    if backward:
        dH = torch.empty_like(H) if dH is None else dH
        dW = torch.empty((V, d), dtype=torch.float32, device=dev) if dW is None else dW
        if dH.shape != H.shape or dW.shape != (V, d):
            raise ValueError("dH / dW have the wrong shape")
    else:
        dH = dW = None
    head = [_dev(H, H.dtype, "H", dev), _dev(W, H.dtype, "W", dev), _dev(tokens, torch.int32, "tokens", dev),
            _dev(logq, torch.float32, "logq", dev), _dev(seq_offsets, torch.int64, "seq_offsets", dev),
            _dev(rewards, torch.float32, "rewards", dev), _dev(group_ids, torch.int32, "group_ids", dev),
            T, d, V, n_seq, n_groups, dt]
    tail = [loss.data_ptr(), logprob.data_ptr(), seq_lr.data_ptr(), vstar.data_ptr(),
            _dev(dH, H.dtype, "dH", dev), _dev(dW, torch.float32, "dW", dev), ws.data_ptr(), ws.numel(),
            _stream(dev)]
    if beta_value is None and not two_pass:
        rc = L.oapl_loss_fwd_bwd(*head, float(beta), float(loss_scale), *tail)
        where = "oapl_loss_fwd_bwd"
    else:
        rc = L.oapl_loss_fwd_bwd_two_beta(*head, float(beta if beta_value is None else beta_value), float(beta),
                                          float(loss_scale), OAPL_FLAG_TWO_PASS if two_pass else 0, *tail)
        where = "oapl_loss_fwd_bwd_two_beta"
    if rc != 0:
        raise OaplError(rc, where)
    return LossResult(loss, logprob, seq_lr, vstar, dH, dW, ws)


def loss_fwd_bwd_noalloc(H, W, tokens, logq, seq_offsets, rewards, group_ids, n_groups: int, beta: float,
                         loss: torch.Tensor, logprob: torch.Tensor, seq_logratio: torch.Tensor, vstar: torch.Tensor,
                         dH: Optional[torch.Tensor], dW: Optional[torch.Tensor], *, loss_scale: float = 1.0) -> None:
    """oapl_loss_fwd_bwd_noalloc: every output is passed in; neither this wrapper nor the library allocates."""
    _check_device(H)
    dt = _dtype_code(H)
    T, d = H.shape
    V = W.shape[0]
    n_seq = rewards.shape[0]
    if W.shape[1] != d or tokens.shape != (T,) or logq.shape != (T,) or seq_offsets.shape != (n_seq + 1,) \
            or group_ids.shape != (n_seq,) or loss.shape != (1,) or logprob.shape != (T,) \
            or seq_logratio.shape != (n_seq,) or vstar.shape != (n_groups,):
        raise ValueError("shape mismatch between the arguments")
    if (dH is None) != (dW is None) or (dH is not None and (dH.shape != H.shape or dW.shape != (V, d))):
        raise ValueError("dH / dW must come as a pair of the right shapes")
    dev = H.device
    rc = lib().oapl_loss_fwd_bwd_noalloc(
        _dev(H, H.dtype, "H", dev), _dev(W, H.dtype, "W", dev), _dev(tokens, torch.int32, "tokens", dev),
        _dev(logq, torch.float32, "logq", dev), _dev(seq_offsets, torch.int64, "seq_offsets", dev),
        _dev(rewards, torch.float32, "rewards", dev), _dev(group_ids, torch.int32, "group_ids", dev),
        T, d, V, n_seq, n_groups, dt, float(beta), float(loss_scale),
        _dev(loss, torch.float32, "loss", dev), _dev(logprob, torch.float32, "logprob", dev),
        _dev(seq_logratio, torch.float32, "seq_logratio", dev), _dev(vstar, torch.float32, "vstar", dev),
        _dev(dH, H.dtype, "dH", dev), _dev(dW, torch.float32, "dW", dev), _stream(dev))
    if rc != 0:
        raise OaplError(rc, "oapl_loss_fwd_bwd_noalloc")


class GrpoResult(NamedTuple):
    loss: torch.Tensor            # [1] float32
    logprob: torch.Tensor         # [T] float32
    advantages: torch.Tensor      # [N] float32
    dH: Optional[torch.Tensor]
    dW: Optional[torch.Tensor]
    workspace: torch.Tensor


def grpo_loss_fwd_bwd(H, W, tokens, logq, logp_old, seq_offsets, rewards, group_ids, n_groups: int, *,
                      clip_eps: float = 0.2, adv_eps: float = 1e-6, loss_scale: float = 1.0, backward: bool = True,
                      two_pass: bool = False, max_panel_rows: Optional[int] = None,
                      max_rollout_len: Optional[int] = None, workspace: Optional[torch.Tensor] = None,
                      dH: Optional[torch.Tensor] = None, dW: Optional[torch.Tensor] = None) -> GrpoResult:
    """oapl_grpo_loss_fwd_bwd: the paper's GRPO + token-level importance sampling baseline."""
    _check_device(H)
    dt = _dtype_code(H)
    T, d = H.shape
    V = W.shape[0]
    n_seq = rewards.shape[0]
    if W.shape[1] != d or tokens.shape != (T,) or logq.shape != (T,) or logp_old.shape != (T,) \
            or seq_offsets.shape != (n_seq + 1,) or group_ids.shape != (n_seq,):
        raise ValueError("shape mismatch between the inputs")
    dev = H.device
    nbytes = workspace_bytes(T, d, V, n_seq, n_groups, dt, backward, max_panel_rows, max_rollout_len)
    if nbytes == 0:
        raise OaplError(2, "oapl_workspace_bytes")
    ws = _workspace(nbytes, dev, workspace)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    logprob = torch.empty(T, dtype=torch.float32, device=dev)
    adv = torch.empty(n_seq, dtype=torch.float32, device=dev)
    if backward:
        dH = torch.empty_like(H) if dH is None else dH
        dW = torch.empty((V, d), dtype=torch.float32, device=dev) if dW is None else dW
        if dH.shape != H.shape or dW.shape != (V, d):
            raise ValueError("dH / dW have the wrong shape")
    else:
        dH = dW = None
    rc = lib().oapl_grpo_loss_fwd_bwd(
        _dev(H, H.dtype, "H", dev), _dev(W, H.dtype, "W", dev), _dev(tokens, torch.int32, "tokens", dev),
        _dev(logq, torch.float32, "logq", dev), _dev(logp_old, torch.float32, "logp_old", dev),
        _dev(seq_offsets, torch.int64, "seq_offsets", dev), _dev(rewards, torch.float32, "rewards", dev),
        _dev(group_ids, torch.int32, "group_ids", dev), T, d, V, n_seq, n_groups, dt, float(clip_eps), float(adv_eps),
        float(loss_scale), OAPL_FLAG_TWO_PASS if two_pass else 0, loss.data_ptr(), logprob.data_ptr(), adv.data_ptr(),
        _dev(dH, H.dtype, "dH", dev),
        _dev(dW, torch.float32, "dW", dev), ws.data_ptr(), ws.numel(), _stream(dev))
    if rc != 0:
        raise OaplError(rc, "oapl_grpo_loss_fwd_bwd")
    return GrpoResult(loss, logprob, adv, dH, dW, ws)


def segmented_sum_f32(x: torch.Tensor, seq_offsets: torch.Tensor) -> torch.Tensor:
    """oapl_segmented_sum_f32: per-rollout sums in double."""
    dev = x.device
    n_seq = seq_offsets.shape[0] - 1
    out = torch.empty(n_seq, dtype=torch.float64, device=dev)
    rc = lib().oapl_segmented_sum_f32(_dev(x, torch.float32, "x", dev), _dev(seq_offsets, torch.int64, "seq_offsets", dev),
                                      n_seq, out.data_ptr(), _stream(dev))
    if rc != 0:
        raise OaplError(rc, "oapl_segmented_sum_f32")
    return out


def timing_enable(on: bool) -> None:
    rc = lib().oapl_timing_enable(1 if on else 0)
    if rc != 0:
        raise OaplError(rc, "oapl_timing_enable")


def timing_read():
    """{kernel name: (total milliseconds, launches)} since timing was enabled."""
    out = {}
    for i, name in enumerate(DENSE_KERNELS):
        ms = ctypes.c_double(0.0)
        n = ctypes.c_int64(0)
        rc = lib().oapl_timing_read(i, ctypes.byref(ms), ctypes.byref(n))
        if rc != 0:
            raise OaplError(rc, "oapl_timing_read")
        out[name] = (float(ms.value), int(n.value))
    return out
