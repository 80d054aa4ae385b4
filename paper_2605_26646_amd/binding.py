"""ctypes binding of libumas.so (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

PLACE_LAST, PLACE_ALL = 0, 1
SEG_TURN, SEG_TRAJ = 0, 1
UMAS_F32, UMAS_BF16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))


class UmasError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libumas status {code}: {message}")
        self.code = code


class _Graph(C.Structure):
    _fields_ = [("n_roles", C.c_int32), ("n_models", C.c_int32), ("n_traj", C.c_int32), ("n_turns", C.c_int32),
                ("n_tokens", C.c_int64), ("role_to_model", C.c_void_p), ("traj_turn_off", C.c_void_p),
                ("turn_role", C.c_void_p), ("turn_tok_off", C.c_void_p), ("turn_pred_off", C.c_void_p),
                ("turn_pred", C.c_void_p), ("traj_group", C.c_void_p)]


class _Rewards(C.Structure):
    _fields_ = [("role_reward", C.c_void_p), ("turn_reward", C.c_void_p), ("traj_reward", C.c_void_p),
                ("w_role", C.c_void_p), ("w_turn", C.c_void_p), ("w_traj", C.c_void_p),
                ("place_mode", C.c_int32), ("norm_eps", C.c_float)]


_STREAM_FIELDS = ["model_tok_off", "perm", "tok_turn", "tok_role", "tok_mask", "tok_reward", "turn_seg_off",
                  "seg_turn", "model_turn_off", "traj_seg_off", "model_trajrun_off", "rowsel",
                  "model_rowsel_off", "turn_scalar", "turn_step", "tok_flags"]


class _Streams(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in _STREAM_FIELDS]


STATS_DTYPE = np.dtype([("loss", "<f4"), ("clip_frac", "<f4"), ("entropy_mean", "<f4"), ("approx_kl", "<f4"),
                        ("n_scored", "<i8"), ("n_invalid_ids", "<i8")])


@dataclass
class Streams:
    """Device tensors written by umas_assign_token_rewards (model-local order)."""
    n_tokens: int
    n_turns: int
    n_models: int
    model_tok_off: torch.Tensor
    perm: torch.Tensor
    tok_turn: torch.Tensor
    tok_role: torch.Tensor
    tok_mask: torch.Tensor
    tok_reward: torch.Tensor
    turn_seg_off: torch.Tensor
    seg_turn: torch.Tensor
    model_turn_off: torch.Tensor
    traj_seg_off: torch.Tensor
    model_trajrun_off: torch.Tensor
    rowsel: torch.Tensor
    model_rowsel_off: torch.Tensor
    turn_scalar: torch.Tensor
    turn_step: torch.Tensor
    tok_flags: torch.Tensor

    def _c(self) -> _Streams:
        s = _Streams()
        for name in _STREAM_FIELDS:
            t = getattr(self, name)
            # an empty tensor has no storage; the ABI wants non-NULL pointers even for size 0
            setattr(s, name, t.data_ptr() or _dummy(t.device).data_ptr())
        return s


_LIB = None
_DUMMY = {}


def _dummy(device) -> torch.Tensor:
    key = str(device)
    if key not in _DUMMY:
        _DUMMY[key] = torch.zeros(256, dtype=torch.uint8, device=device)
    return _DUMMY[key]


def lib_path() -> str:
    return os.path.join(_HERE, "libumas.so")


def load_library():
    """Load libumas.so built in-tree; there is no fallback when it is missing."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(path)
    lib.umas_last_error.restype = C.c_char_p
    for name in ("umas_assign_workspace_bytes", "umas_advantages_workspace_bytes",
                 "umas_policy_logprobs_workspace_bytes", "umas_ppo_loss_workspace_bytes",
                 "umas_ppo_loss_workspace_bytes_min"):
        getattr(lib, name).restype = C.c_size_t
    lib.umas_assign_workspace_bytes.argtypes = [C.c_void_p]
    lib.umas_advantages_workspace_bytes.argtypes = [C.c_int64]
    lib.umas_policy_logprobs_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int]
    lib.umas_ppo_loss_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int, C.c_int32]
    lib.umas_ppo_loss_workspace_bytes_min.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int, C.c_int32]
    lib.umas_assign_token_rewards.restype = C.c_int
    lib.umas_assign_token_rewards.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_size_t, C.c_void_p]
    lib.umas_advantages.restype = C.c_int
    lib.umas_advantages.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_float, C.c_float, C.c_float,
                                    C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.umas_policy_logprobs.restype = C.c_int
    lib.umas_policy_logprobs.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_int32,
                                         C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
    lib.umas_ppo_loss_fwd_bwd.restype = C.c_int
    lib.umas_ppo_loss_fwd_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_int32,
                                          C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_int32, C.c_float, C.c_float, C.c_float, C.c_int32, C.c_int64, C.c_void_p,
                                          C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                          C.c_void_p]
    _LIB = lib
    return lib


def _check(lib, status: int):
    if status != 0:
        raise UmasError(status, lib.umas_last_error().decode())


def _host(arr, dtype):
    """Contiguous host array of the ABI's type, or None; returns (array kept alive, pointer)."""
    if arr is None:
        return None, None
    a = np.ascontiguousarray(arr, dtype=dtype)
    return a, a.ctypes.data


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _sel_ptr(rowsel: Optional[torch.Tensor]):
    """Pointer of a row selection; an empty selection still needs a non-NULL pointer (NULL means all rows)."""
    if rowsel is None:
        return None, None
    if rowsel.numel() == 0:
        dummy = torch.zeros(1, dtype=torch.int32, device=rowsel.device)
        return dummy, dummy.data_ptr()
    return rowsel, rowsel.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


# Row selections are device data that the library cannot check.  With CHECK_ROWS on (the test suite switches it on)
# every call that takes one first reads its range back and refuses entries outside [0, n_rows): a mistake in a caller
# then raises here instead of sending a kernel out of bounds.  It waits for the stream, so it stays off by default
# and is skipped under graph capture.
CHECK_ROWS = False


def _check_rows(rowsel: Optional[torch.Tensor], n_rows: int):
    if not CHECK_ROWS or rowsel is None or rowsel.numel() == 0 or torch.cuda.is_current_stream_capturing():
        return
    lo, hi = int(rowsel.min().item()), int(rowsel.max().item())
    if lo < 0 or hi >= n_rows:
        raise UmasError(-1, f"row selection holds entries from {lo} to {hi}, outside [0, {n_rows})")


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return UMAS_F32
    if t.dtype == torch.bfloat16:
        return UMAS_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def umas_assign_token_rewards(*, n_roles, n_models, role_to_model, traj_turn_off, turn_role, turn_tok_off,
                              tok_mask_global: torch.Tensor, turn_pred_off=None, turn_pred=None, traj_group=None,
                              role_reward=None, turn_reward=None, traj_reward=None, w_role=None, w_turn=None,
                              w_traj=None, place_mode=PLACE_LAST, norm_eps=1e-6) -> Streams:
    lib = load_library()
    keep = []

    def h(a, dt):
        arr, p = _host(a, dt)
        keep.append(arr)
        return p

    traj_turn_off = np.asarray(traj_turn_off)
    turn_tok_off = np.asarray(turn_tok_off)
    n_traj, n_turns = len(traj_turn_off) - 1, len(turn_tok_off) - 1
    n_tokens = int(tok_mask_global.numel())
    g = _Graph(n_roles, n_models, n_traj, n_turns, n_tokens, h(role_to_model, np.int32), h(traj_turn_off, np.int32),
               h(turn_role, np.int32), h(turn_tok_off, np.int64), h(turn_pred_off, np.int32), h(turn_pred, np.int32),
               h(traj_group, np.int32))
    r = _Rewards(h(role_reward, np.float32), h(turn_reward, np.float32), h(traj_reward, np.float32),
                 h(w_role, np.float32), h(w_turn, np.float32), h(w_traj, np.float32), place_mode, norm_eps)
    dev = tok_mask_global.device
    i64 = dict(dtype=torch.int64, device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    out = Streams(
        n_tokens=n_tokens, n_turns=n_turns, n_models=n_models,
        model_tok_off=torch.empty(n_models + 1, **i64), perm=torch.empty(n_tokens, **i64),
        tok_turn=torch.empty(n_tokens, **i32), tok_role=torch.empty(n_tokens, **i32),
        tok_mask=torch.empty(n_tokens, dtype=torch.uint8, device=dev), tok_reward=torch.empty(n_tokens, **f32),
        turn_seg_off=torch.empty(n_turns + 1, **i64), seg_turn=torch.empty(max(n_turns, 1), **i32),
        model_turn_off=torch.empty(n_models + 1, **i32), traj_seg_off=torch.empty(n_turns + 1, **i64),
        model_trajrun_off=torch.empty(n_models + 1, **i32), rowsel=torch.empty(max(n_tokens, 1), **i32),
        model_rowsel_off=torch.empty(n_models + 1, **i64), turn_scalar=torch.empty(max(n_turns, 1), **f32),
        turn_step=torch.empty(max(n_turns, 1), **i32),
        tok_flags=torch.empty(n_tokens, dtype=torch.uint8, device=dev))
    ws = _workspace(lib.umas_assign_workspace_bytes(C.addressof(g)), dev)
    cs = out._c()
    _check(lib, lib.umas_assign_token_rewards(C.addressof(g), C.addressof(r), _ptr(tok_mask_global) or _dummy(dev).data_ptr(), C.addressof(cs),
                                              ws.data_ptr(), ws.numel(), _stream()))
    return out


def umas_advantages(streams: Streams, value: Optional[torch.Tensor], gamma, lam, gamma_turn=1.0, seg_mode=SEG_TURN):
    lib = load_library()
    dev = streams.tok_reward.device
    adv = torch.empty(streams.n_tokens, dtype=torch.float32, device=dev)
    ret = torch.empty(streams.n_tokens, dtype=torch.float32, device=dev)
    ws = _workspace(lib.umas_advantages_workspace_bytes(streams.n_tokens), dev)
    cs = streams._c()
    _check(lib, lib.umas_advantages(C.addressof(cs), streams.n_tokens, streams.n_turns, _ptr(value), gamma, lam,
                                    gamma_turn, seg_mode, adv.data_ptr(), ret.data_ptr(), ws.data_ptr(), ws.numel(),
                                    _stream()))
    return adv, ret


def umas_policy_logprobs(H: torch.Tensor, W: torch.Tensor, ids: torch.Tensor, rowsel: Optional[torch.Tensor] = None,
                         want_entropy=True, workspace: Optional[torch.Tensor] = None):
    lib = load_library()
    n_rows, d = H.shape
    V = W.shape[0]
    n_sel = n_rows if rowsel is None else int(rowsel.numel())
    dt = _dtype_code(H)
    dev = H.device
    logp = torch.empty(n_rows, dtype=torch.float32, device=dev)
    lse = torch.empty(n_rows, dtype=torch.float32, device=dev)
    ent = torch.empty(n_rows, dtype=torch.float32, device=dev) if want_entropy else None
    ws = workspace if workspace is not None else _workspace(lib.umas_policy_logprobs_workspace_bytes(n_sel, d, V, dt), dev)
    _check_rows(rowsel, n_rows)
    _keep, sel = _sel_ptr(rowsel)
    _check(lib, lib.umas_policy_logprobs(H.data_ptr(), W.data_ptr(), dt, n_rows, d, V, ids.data_ptr(), sel,
                                         n_sel, logp.data_ptr(), lse.data_ptr(), _ptr(ent), ws.data_ptr(), ws.numel(),
                                         _stream()))
    return logp, lse, ent


STATIC_SCRATCH_BYTES = 32 << 20


def umas_policy_logprobs_static(H: torch.Tensor, W: torch.Tensor, ids: torch.Tensor, rowsel: Optional[torch.Tensor] = None,
                                logp=None, lse=None, entropy=None):
    """umas_policy_logprobs without a workspace (the library's static scratch); the outputs may be passed in, so that
    the call itself allocates nothing."""
    lib = load_library()
    lib.umas_policy_logprobs_static.restype = C.c_int
    lib.umas_policy_logprobs_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_int32,
                                                C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_void_p]
    n_rows, d = H.shape
    V = W.shape[0]
    n_sel = n_rows if rowsel is None else int(rowsel.numel())
    dev = H.device
    if logp is None:
        logp = torch.empty(n_rows, dtype=torch.float32, device=dev)
    if lse is None:
        lse = torch.empty(n_rows, dtype=torch.float32, device=dev)
    if entropy is None:
        entropy = torch.empty(n_rows, dtype=torch.float32, device=dev)
    _check_rows(rowsel, n_rows)
    _keep, sel = _sel_ptr(rowsel)
    _check(lib, lib.umas_policy_logprobs_static(H.data_ptr(), W.data_ptr(), _dtype_code(H), n_rows, d, V, ids.data_ptr(),
                                                sel, n_sel, logp.data_ptr(), lse.data_ptr(), entropy.data_ptr(), _stream()))
    return logp, lse, entropy


def ppo_workspace_bytes(n_sel, d, V, dtype: torch.dtype, n_roles, minimum=False) -> int:
    lib = load_library()
    code = UMAS_BF16 if dtype == torch.bfloat16 else UMAS_F32
    f = lib.umas_ppo_loss_workspace_bytes_min if minimum else lib.umas_ppo_loss_workspace_bytes
    return int(f(n_sel, d, V, code, n_roles))


def umas_ppo_loss_fwd_bwd(H, W, ids, rowsel, logp_old, adv, tok_role, n_roles, clip_eps, *, entropy_coef=0.0,
                          dual_clip=0.0, accumulate_dW=False, norm_rows=0, logp_ref=None, kl_coef=0.0, dW=None, dH=None,
                          logp_new=None, stats=None, workspace=None):
    lib = load_library()
    n_rows, d = H.shape
    V = W.shape[0]
    n_sel = n_rows if rowsel is None else int(rowsel.numel())
    dt = _dtype_code(H)
    dev = H.device
    if dW is None:
        dW = torch.empty((V, d), dtype=torch.float32, device=dev)
    if dH is None:
        dH = torch.empty_like(H)
    if logp_new is None:
        logp_new = torch.empty(n_rows, dtype=torch.float32, device=dev)
    if stats is None:
        stats = torch.empty((1 + n_roles) * STATS_DTYPE.itemsize, dtype=torch.uint8, device=dev)
    ws = workspace if workspace is not None else _workspace(
        lib.umas_ppo_loss_workspace_bytes(n_sel, d, V, dt, n_roles), dev)
    _check_rows(rowsel, n_rows)
    _keep, sel = _sel_ptr(rowsel)
    _check(lib, lib.umas_ppo_loss_fwd_bwd(H.data_ptr(), W.data_ptr(), dt, n_rows, d, V, ids.data_ptr(), sel,
                                          n_sel, _ptr(logp_old), adv.data_ptr(), _ptr(tok_role), n_roles,
                                          clip_eps, entropy_coef, dual_clip, 1 if accumulate_dW else 0, int(norm_rows),
                                          _ptr(logp_ref), kl_coef, stats.data_ptr(),
                                          logp_new.data_ptr(), dH.data_ptr(), dW.data_ptr(), ws.data_ptr(), ws.numel(),
                                          _stream()))
    return stats, logp_new, dH, dW


VALUE_STATS_DTYPE = np.dtype([("loss", "<f4"), ("clip_frac", "<f4"), ("value_mean", "<f4"), ("reserved", "<f4"),
                              ("n_scored", "<i8")])


def umas_values(H, w, bias=0.0, rowsel=None, value=None):
    lib = load_library()
    lib.umas_values.restype = C.c_int
    lib.umas_values.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int, C.c_int64, C.c_int32, C.c_void_p, C.c_int64,
                                C.c_void_p, C.c_void_p]
    n_rows, d = H.shape
    n_sel = n_rows if rowsel is None else int(rowsel.numel())
    if value is None:
        value = torch.empty(n_rows, dtype=torch.float32, device=H.device)
    _check_rows(rowsel, n_rows)
    _keep, sel = _sel_ptr(rowsel)
    _check(lib, lib.umas_values(_ptr(H), w.data_ptr(), bias, _dtype_code(H), n_rows, d, sel, n_sel, _ptr(value), _stream()))
    return value


def umas_value_loss_fwd_bwd(H, w, bias, rowsel, value_old, ret, tok_role, n_roles, clip_eps_v, *, accumulate_dH=False,
                            accumulate_dw=False, norm_rows=0, dH=None, dw=None, db=None, value_new=None, stats=None,
                            workspace=None):
    lib = load_library()
    lib.umas_value_workspace_bytes.restype = C.c_size_t
    lib.umas_value_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int, C.c_int32]
    lib.umas_value_loss_fwd_bwd.restype = C.c_int
    lib.umas_value_loss_fwd_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int, C.c_int64, C.c_int32, C.c_void_p,
                                            C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_int32,
                                            C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_size_t, C.c_void_p]
    n_rows, d = H.shape
    n_sel = n_rows if rowsel is None else int(rowsel.numel())
    dt = _dtype_code(H)
    dev = H.device
    if dH is None:
        dH = torch.empty_like(H)
    if dw is None:
        dw = torch.empty(d, dtype=torch.float32, device=dev)
    if db is None:
        db = torch.empty(1, dtype=torch.float32, device=dev)
    if value_new is None:
        value_new = torch.empty(n_rows, dtype=torch.float32, device=dev)
    if stats is None:
        stats = torch.empty((1 + n_roles) * VALUE_STATS_DTYPE.itemsize, dtype=torch.uint8, device=dev)
    ws = workspace if workspace is not None else _workspace(lib.umas_value_workspace_bytes(n_sel, d, dt, n_roles), dev)
    _check_rows(rowsel, n_rows)
    _keep, sel = _sel_ptr(rowsel)
    _check(lib, lib.umas_value_loss_fwd_bwd(_ptr(H), w.data_ptr(), bias, dt, n_rows, d, sel, n_sel, _ptr(value_old),
                                            _ptr(ret), _ptr(tok_role), n_roles, clip_eps_v, 1 if accumulate_dH else 0,
                                            1 if accumulate_dw else 0, int(norm_rows), stats.data_ptr(), _ptr(value_new), _ptr(dH),
                                            dw.data_ptr(), db.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return stats, value_new, dH, dw, db


WHITEN_MODEL, WHITEN_MODEL_ROLE = 0, 1


def umas_kl_rewards(tok_reward, logp, logp_ref, tok_mask, beta, out=None):
    """Returns (penalised rewards, device float[1] mean of logp - logp_ref over the mask=1 tokens)."""
    lib = load_library()
    lib.umas_kl_rewards_workspace_bytes.restype = C.c_size_t
    lib.umas_kl_rewards_workspace_bytes.argtypes = [C.c_int64]
    lib.umas_kl_rewards.restype = C.c_int
    lib.umas_kl_rewards.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    n = int(tok_reward.numel())
    dev = tok_reward.device
    if out is None:
        out = torch.empty_like(tok_reward)
    kl = torch.empty(1, dtype=torch.float32, device=dev)
    ws = _workspace(lib.umas_kl_rewards_workspace_bytes(n), dev)
    d = _dummy(dev).data_ptr()
    p = (lambda t: t.data_ptr() if n else d)
    _check(lib, lib.umas_kl_rewards(p(tok_reward), p(logp), p(logp_ref), p(tok_mask), n, beta, p(out), kl.data_ptr(),
                                    ws.data_ptr(), ws.numel(), _stream()))
    return out, kl


def umas_whiten_advantages(adv, tok_mask, tok_role, model_tok_off, n_roles, scope=WHITEN_MODEL, eps=1e-8, out=None):
    lib = load_library()
    lib.umas_whiten_workspace_bytes.restype = C.c_size_t
    lib.umas_whiten_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
    lib.umas_whiten_advantages.restype = C.c_int
    lib.umas_whiten_advantages.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int64,
                                           C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    n = int(adv.numel())
    dev = adv.device
    off_keep, off_ptr = _host(model_tok_off, np.int64)
    n_models = len(off_keep) - 1
    if out is None:
        out = torch.empty_like(adv)
    ws = _workspace(lib.umas_whiten_workspace_bytes(n, n_models, n_roles), dev)
    d = _dummy(dev).data_ptr()
    p = (lambda t: None if t is None else (t.data_ptr() if n else d))
    _check(lib, lib.umas_whiten_advantages(p(adv), p(tok_mask), p(tok_role), off_ptr, n_models, n_roles, n, scope, eps,
                                           p(out), ws.data_ptr(), ws.numel(), _stream()))
    return out


def umas_ready_batch(streams: Streams, traj_turn_off, n_minibatch, traj_keep=None, traj_order=None, balance_rows=False):
    """Returns (mb_rowsel device int32, mb_off device int64 [n_models, n_minibatch + 1]); balance_rows selects
    umas_ready_batch_balanced (parts cut by scored rows per model instead of by trajectories)."""
    lib = load_library()
    lib.umas_ready_batch_workspace_bytes.restype = C.c_size_t
    lib.umas_ready_batch_workspace_bytes.argtypes = [C.c_int32, C.c_int32]
    fn = lib.umas_ready_batch_balanced if balance_rows else lib.umas_ready_batch
    fn.restype = C.c_int
    fn.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                   C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    dev = streams.rowsel.device
    tto_keep, tto = _host(traj_turn_off, np.int32)
    n_traj = len(tto_keep) - 1
    keep_keep, keep = _host(traj_keep, np.uint8)
    order_keep, order = _host(traj_order, np.int32)
    mb_rowsel = torch.empty(max(int(streams.rowsel.numel()), 1), dtype=torch.int32, device=dev)
    mb_off = torch.empty((streams.n_models, n_minibatch + 1), dtype=torch.int64, device=dev)
    ws = _workspace(lib.umas_ready_batch_workspace_bytes(n_traj, streams.n_models), dev)
    cs = streams._c()
    _check(lib, fn(C.addressof(cs), streams.n_models, streams.n_turns, tto, n_traj, keep, order,
                   n_minibatch, mb_rowsel.data_ptr(), mb_off.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return mb_rowsel, mb_off


def umas_ready_batch_packed(streams: Streams, traj_turn_off, max_rows, traj_keep=None, traj_order=None):
    """Returns (mb_rowsel device int32, mb_off device int64 [n_models, n_traj + 1], n_parts device int32 [n_models]):
    micro-batches of whole trajectories under a budget of max_rows scored rows."""
    lib = load_library()
    lib.umas_ready_batch_workspace_bytes.restype = C.c_size_t
    lib.umas_ready_batch_workspace_bytes.argtypes = [C.c_int32, C.c_int32]
    fn = lib.umas_ready_batch_packed
    fn.restype = C.c_int
    fn.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                   C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    dev = streams.rowsel.device
    tto_keep, tto = _host(traj_turn_off, np.int32)
    n_traj = len(tto_keep) - 1
    keep_keep, keep = _host(traj_keep, np.uint8)
    order_keep, order = _host(traj_order, np.int32)
    mb_rowsel = torch.empty(max(int(streams.rowsel.numel()), 1), dtype=torch.int32, device=dev)
    mb_off = torch.empty((streams.n_models, n_traj + 1), dtype=torch.int64, device=dev)
    n_parts = torch.empty(streams.n_models, dtype=torch.int32, device=dev)
    ws = _workspace(lib.umas_ready_batch_workspace_bytes(n_traj, streams.n_models), dev)
    cs = streams._c()
    _check(lib, fn(C.addressof(cs), streams.n_models, streams.n_turns, tto, n_traj, keep, order, int(max_rows),
                   mb_rowsel.data_ptr(), mb_off.data_ptr(), n_parts.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return mb_rowsel, mb_off, n_parts


def read_value_stats(stats: torch.Tensor) -> np.ndarray:
    return stats.cpu().numpy().view(VALUE_STATS_DTYPE)


def read_stats(stats: torch.Tensor) -> np.ndarray:
    """Copy the device umas_loss_stats array to a numpy structured array (synchronises)."""
    return stats.cpu().numpy().view(STATS_DTYPE)


def profile_enable(on: bool) -> None:
    """Switch the library's per-kernel event timing on (discarding earlier records) or off."""
    lib = load_library()
    lib.umas_profile_enable.restype = C.c_int
    lib.umas_profile_enable.argtypes = [C.c_int32]
    _check(lib, lib.umas_profile_enable(1 if on else 0))


def profile_read(cap: int = 64) -> dict:
    """{kernel name: (total milliseconds, launches)} since profile_enable(True); synchronises."""
    lib = load_library()
    lib.umas_profile_read.restype = C.c_int32
    lib.umas_profile_read.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
    names = C.create_string_buffer(32 * cap)
    ms = (C.c_float * cap)()
    cnt = (C.c_int32 * cap)()
    n = lib.umas_profile_read(names, ms, cnt, cap)
    if n < 0:
        raise UmasError(-5, "umas_profile_read failed")
    out = {}
    for i in range(n):
        out[names.raw[32 * i:32 * i + 32].split(b"\0")[0].decode()] = (float(ms[i]), int(cnt[i]))
    return out
