"""Thin ctypes binding over libprefix_attn.so (the C ABI in include/prefix_attn.h).

Argument marshalling only: every step of the attention runs in the library's HIP
kernels.  PyTorch tensors are used as device memory; the binding passes raw
device pointers and the current HIP stream.  There is no CPU fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libprefix_attn.so")
_lib = None

PA_F32, PA_BF16 = 0, 1
STATUS_NAMES = {0: "PA_OK", 1: "PA_ERR_NULL", 2: "PA_ERR_SHAPE", 3: "PA_ERR_UNSUPPORTED", 4: "PA_ERR_ALIGN",
                5: "PA_ERR_WORKSPACE", 6: "PA_ERR_ALLOC", 7: "PA_ERR_HIP"}
STATIC_SCRATCH_BYTES = 64 << 20      # PA_STATIC_SCRATCH_BYTES of the header
EXPORTED_SYMBOLS = ("prefix_attn_plan", "prefix_attn_forward", "prefix_attn_forward_static", "prefix_attn_forward_timed", "prefix_attn_lse", "prefix_attn_destroy",
                    "prefix_attn_status_string", "prefix_attn_plan_tiles", "prefix_attn_plan_num_items",
                    "prefix_attn_plan_items", "prefix_attn_plan_total_tokens", "prefix_attn_backward_workspace",
                    "prefix_attn_backward", "prefix_attn_backward_timed", "prefix_attn_plan_num_key_items",
                    "prefix_attn_plan_key_items", "prefix_attn_plan_key_item_extra_tiles", "prefix_attn_forward_partial", "prefix_attn_merge_partials")
EXPORTED_SYMBOLS_OTHER = ("token_logprob_workspace", "token_logprob_forward", "grpo_group_advantages")


class PrefixAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().prefix_attn_status_string(status).decode()
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({msg})")


class _Desc(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("prefix_len", ctypes.c_int64), ("num_rollouts", ctypes.c_int32),
                ("suffix_lens", ctypes.POINTER(ctypes.c_int32)), ("softmax_scale", ctypes.c_float),
                ("dtype", ctypes.c_int32), ("device", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the C-ABI library; raises if it has not been built (python -m paper_2507_07966_amd.build).

    torch is imported first: it carries its own copy of the HIP runtime under the same soname, and the
    tensors whose device pointers the calls receive live in that runtime.  Loading this library before
    torch would bring in the system's copy as a second runtime in the process, whose allocations fail."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} is missing: build it with `python -m paper_2507_07966_amd.build`")
    import torch  # noqa: F401  (see above)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    lib.prefix_attn_plan.restype = ctypes.c_int
    lib.prefix_attn_plan.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(vp), ctypes.POINTER(sz)]
    lib.prefix_attn_forward.restype = ctypes.c_int
    lib.prefix_attn_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.prefix_attn_forward_static.restype = ctypes.c_int
    lib.prefix_attn_forward_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.prefix_attn_forward_timed.restype = ctypes.c_int
    lib.prefix_attn_forward_timed.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, ctypes.POINTER(ctypes.c_float)]
    lib.prefix_attn_lse.restype = ctypes.c_int
    lib.prefix_attn_lse.argtypes = [vp, vp, vp, vp]
    lib.prefix_attn_destroy.restype = None
    lib.prefix_attn_destroy.argtypes = [vp]
    lib.prefix_attn_status_string.restype = ctypes.c_char_p
    lib.prefix_attn_status_string.argtypes = [ctypes.c_int]
    lib.prefix_attn_plan_tiles.restype = ctypes.c_int
    lib.prefix_attn_plan_tiles.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    lib.prefix_attn_plan_num_items.restype = ctypes.c_int64
    lib.prefix_attn_plan_num_items.argtypes = [vp, ctypes.c_int32]
    lib.prefix_attn_plan_items.restype = ctypes.c_int
    lib.prefix_attn_plan_items.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    lib.prefix_attn_plan_total_tokens.restype = ctypes.c_int64
    lib.prefix_attn_plan_total_tokens.argtypes = [vp]
    lib.prefix_attn_forward_partial.restype = ctypes.c_int
    lib.prefix_attn_forward_partial.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp, vp, vp, sz, vp]
    lib.prefix_attn_merge_partials.restype = ctypes.c_int
    lib.prefix_attn_merge_partials.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp, vp]
    lib.token_logprob_workspace.restype = ctypes.c_int
    lib.token_logprob_workspace.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(sz)]
    lib.token_logprob_forward.restype = ctypes.c_int
    lib.token_logprob_forward.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                          vp, vp, vp, sz, vp]
    lib.grpo_group_advantages.restype = ctypes.c_int
    lib.grpo_group_advantages.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.prefix_attn_backward_workspace.restype = ctypes.c_int
    lib.prefix_attn_backward_workspace.argtypes = [vp, ctypes.POINTER(sz)]
    lib.prefix_attn_backward.restype = ctypes.c_int
    lib.prefix_attn_backward.argtypes = [vp] * 15 + [sz, vp]
    lib.prefix_attn_backward_timed.restype = ctypes.c_int
    lib.prefix_attn_backward_timed.argtypes = [vp] * 15 + [sz, vp, ctypes.POINTER(ctypes.c_float)]
    lib.prefix_attn_plan_num_key_items.restype = ctypes.c_int64
    lib.prefix_attn_plan_num_key_items.argtypes = [vp, ctypes.c_int32]
    lib.prefix_attn_plan_key_items.restype = ctypes.c_int
    lib.prefix_attn_plan_key_items.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    lib.prefix_attn_plan_key_item_extra_tiles.restype = ctypes.c_int
    lib.prefix_attn_plan_key_item_extra_tiles.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    _lib = lib
    return lib


def prefix_attn_status_string(status: int) -> str:
    return load_library().prefix_attn_status_string(int(status)).decode()


class PrefixAttnPlan:
    """Owner of a prefix_attn_plan_t*; see prefix_attn_plan()."""

    def __init__(self, handle, workspace_bytes, desc_kw):
        self._h = handle
        self.workspace_bytes = int(workspace_bytes)
        self.__dict__.update(desc_kw)

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("plan was destroyed")
        return self._h

    @property
    def total_tokens(self) -> int:
        return int(load_library().prefix_attn_plan_total_tokens(self.handle))

    def tiles(self):
        a, b = ctypes.c_int32(), ctypes.c_int32()
        st = load_library().prefix_attn_plan_tiles(self.handle, ctypes.byref(a), ctypes.byref(b))
        if st:
            raise PrefixAttnError(st, "prefix_attn_plan_tiles")
        return a.value, b.value

    def items(self, which: int) -> np.ndarray:
        """Work list of pass 0 (prefix), 1 (suffix), 2 (backward dQ) or 3 (forward single sweep, empty unless used):
        int32 [n, 6] = (g, row0, c, nkeys, key0, pkeys)."""
        lib = load_library()
        n = lib.prefix_attn_plan_num_items(self.handle, which)
        if n < 0:
            raise PrefixAttnError(2, "prefix_attn_plan_num_items")
        out = np.zeros((n, 6), dtype=np.int32)
        if n:
            st = lib.prefix_attn_plan_items(self.handle, which, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
            if st:
                raise PrefixAttnError(st, "prefix_attn_plan_items")
        return out

    @property
    def backward_workspace_bytes(self) -> int:
        n = ctypes.c_size_t()
        st = load_library().prefix_attn_backward_workspace(self.handle, ctypes.byref(n))
        if st:
            raise PrefixAttnError(st, "prefix_attn_backward_workspace")
        return int(n.value)

    def key_item_extra_tiles(self, which: int) -> np.ndarray:
        """int32 [n]: the one row tile an item of dK/dV list `which` streams after [tile0, tile1), or -1."""
        lib = load_library()
        n = lib.prefix_attn_plan_num_key_items(self.handle, which)
        if n < 0:
            raise PrefixAttnError(2, "prefix_attn_plan_num_key_items")
        out = np.full(n, -1, dtype=np.int32)
        if n:
            st = lib.prefix_attn_plan_key_item_extra_tiles(self.handle, which, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
            if st:
                raise PrefixAttnError(st, "prefix_attn_plan_key_item_extra_tiles")
        return out

    def key_items(self, which: int) -> np.ndarray:
        """dK/dV work list, 0 (prefix key blocks), 1 (the rollouts' own key blocks, masked kernel) or 2 (the same
        blocks for the mask-free kernel, empty unless the plan splits that pass): int32 [n, 6] =
        (g, key0, c, nkeys, tile0, tile1); [tile0, tile1) is the range of row tiles the item streams."""
        lib = load_library()
        n = lib.prefix_attn_plan_num_key_items(self.handle, which)
        if n < 0:
            raise PrefixAttnError(2, "prefix_attn_plan_num_key_items")
        out = np.zeros((n, 6), dtype=np.int32)
        if n:
            st = lib.prefix_attn_plan_key_items(self.handle, which, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
            if st:
                raise PrefixAttnError(st, "prefix_attn_plan_key_items")
        return out

    def destroy(self):
        if self._h is not None:
            load_library().prefix_attn_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def prefix_attn_plan(num_q_heads: int, num_kv_heads: int, head_dim: int, prefix_len: int,
                     suffix_lens: Sequence[int], softmax_scale: float, dtype: str = "bf16",
                     device: int = 0) -> PrefixAttnPlan:
    """prefix_attn_plan of the C ABI.  dtype "bf16" | "f32"; device -1 = host-only plan."""
    lib = load_library()
    lens = np.ascontiguousarray(suffix_lens, dtype=np.int32)
    d = _Desc()
    d.num_q_heads, d.num_kv_heads, d.head_dim = int(num_q_heads), int(num_kv_heads), int(head_dim)
    d.prefix_len, d.num_rollouts = int(prefix_len), int(len(lens))
    d.suffix_lens = lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if len(lens) else None
    d.softmax_scale = float(softmax_scale)
    d.dtype = {"f32": PA_F32, "bf16": PA_BF16}.get(dtype, dtype if isinstance(dtype, int) else -1)
    d.device = int(device)
    h, ws = ctypes.c_void_p(), ctypes.c_size_t()
    st = lib.prefix_attn_plan(ctypes.byref(d), ctypes.byref(h), ctypes.byref(ws))
    if st:
        raise PrefixAttnError(st, "prefix_attn_plan")
    kw = dict(num_q_heads=d.num_q_heads, num_kv_heads=d.num_kv_heads, head_dim=d.head_dim, prefix_len=d.prefix_len,
              suffix_lens=lens.copy(), softmax_scale=d.softmax_scale, dtype=dtype, device=d.device)
    return PrefixAttnPlan(h, ws.value, kw)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def prefix_attn_forward(plan: PrefixAttnPlan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, workspace,
                        stream=None) -> None:
    """prefix_attn_forward of the C ABI.  Tensors are torch device tensors (or raw int pointers);
    `workspace` is a uint8 tensor of at least plan.workspace_bytes.  Enqueues only."""
    ws_bytes = workspace.numel() * workspace.element_size() if hasattr(workspace, "numel") else plan.workspace_bytes
    st = load_library().prefix_attn_forward(plan.handle, _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_suffix),
                                            _ptr(v_suffix), _ptr(out), _ptr(workspace), ws_bytes, _stream(stream))
    if st:
        raise PrefixAttnError(st, "prefix_attn_forward")


def prefix_attn_forward_static(plan: PrefixAttnPlan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, lse_out=None,
                               stream=None) -> None:
    """prefix_attn_forward_static of the C ABI: forward (+ LSE export when lse_out is given) on the library's
    own static workspace; for plans of at most STATIC_SCRATCH_BYTES of workspace.  Enqueues only."""
    st = load_library().prefix_attn_forward_static(plan.handle, _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_suffix),
                                                   _ptr(v_suffix), _ptr(out), _ptr(lse_out), _stream(stream))
    if st:
        raise PrefixAttnError(st, "prefix_attn_forward_static")


def prefix_attn_forward_timed(plan: PrefixAttnPlan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, workspace,
                              stream=None):
    """prefix_attn_forward_timed of the C ABI.  Waits; returns (prepass_ms, prefix_ms, suffix_ms, merge_ms)."""
    ws_bytes = workspace.numel() * workspace.element_size() if hasattr(workspace, "numel") else plan.workspace_bytes
    ms = (ctypes.c_float * 4)()
    st = load_library().prefix_attn_forward_timed(plan.handle, _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_suffix),
                                                  _ptr(v_suffix), _ptr(out), _ptr(workspace), ws_bytes,
                                                  _stream(stream), ms)
    if st:
        raise PrefixAttnError(st, "prefix_attn_forward_timed")
    return float(ms[0]), float(ms[1]), float(ms[2]), float(ms[3])


def prefix_attn_forward_partial(plan: PrefixAttnPlan, q, k_prefix, v_prefix, k_suffix, v_suffix, include_suffix: bool,
                                o_partial, lse_partial, workspace, stream=None) -> None:
    """prefix_attn_forward_partial of the C ABI: fp32 partial (o [T,Hq,D], lse [T,Hq]) over this plan's prefix
    shard, plus the rollouts' own keys when include_suffix."""
    st = load_library().prefix_attn_forward_partial(
        plan.handle, _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_suffix), _ptr(v_suffix), int(bool(include_suffix)),
        _ptr(o_partial), _ptr(lse_partial), _ptr(workspace), _nbytes(workspace, plan.workspace_bytes), _stream(stream))
    if st:
        raise PrefixAttnError(st, "prefix_attn_forward_partial")


def prefix_attn_merge_partials(plan: PrefixAttnPlan, o_partials, lse_partials, out, lse_out=None, stream=None) -> None:
    """prefix_attn_merge_partials of the C ABI: combine fp32 partials over disjoint key sets into out (and lse_out [Hq,T])."""
    n = len(o_partials)
    arr = ctypes.c_void_p * max(n, 1)
    st = load_library().prefix_attn_merge_partials(
        plan.handle, n, arr(*[_ptr(t) for t in o_partials]), arr(*[_ptr(t) for t in lse_partials]), _ptr(out),
        _ptr(lse_out), _stream(stream))
    if st:
        raise PrefixAttnError(st, "prefix_attn_merge_partials")


def prefix_attn_lse(plan: PrefixAttnPlan, workspace, lse_out, stream=None) -> None:
    """prefix_attn_lse of the C ABI: merged LSE [Hq, T] fp32 of the last forward on `workspace`."""
    st = load_library().prefix_attn_lse(plan.handle, _ptr(workspace), _ptr(lse_out), _stream(stream))
    if st:
        raise PrefixAttnError(st, "prefix_attn_lse")


def _nbytes(t, default):
    return t.numel() * t.element_size() if hasattr(t, "numel") else default


def _backward_args(plan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, d_out, lse, dq, dk_prefix,
                   dv_prefix, dk_suffix, dv_suffix, workspace, stream):
    return (plan.handle, _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_suffix), _ptr(v_suffix), _ptr(out),
            _ptr(d_out), _ptr(lse), _ptr(dq), _ptr(dk_prefix), _ptr(dv_prefix), _ptr(dk_suffix),
            _ptr(dv_suffix), _ptr(workspace), _nbytes(workspace, plan.backward_workspace_bytes), _stream(stream))


def prefix_attn_backward(plan: PrefixAttnPlan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, d_out,
                         lse, dq, dk_prefix, dv_prefix, dk_suffix, dv_suffix, workspace,
                         stream=None) -> None:
    """prefix_attn_backward of the C ABI.  `lse` is the [Hq, T] fp32 tensor written by prefix_attn_lse after the forward call on the
    same inputs; `workspace` is a uint8 tensor of at least plan.backward_workspace_bytes.  Enqueues only."""
    st = load_library().prefix_attn_backward(*_backward_args(
        plan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, d_out, lse, dq, dk_prefix, dv_prefix,
        dk_suffix, dv_suffix, workspace, stream))
    if st:
        raise PrefixAttnError(st, "prefix_attn_backward")


def prefix_attn_backward_timed(plan: PrefixAttnPlan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, d_out,
                               lse, dq, dk_prefix, dv_prefix, dk_suffix, dv_suffix, workspace,
                               stream=None):
    """prefix_attn_backward_timed of the C ABI.  Waits; returns (prepass_ms, dq_ms, dkv_prefix_ms, dkv_suffix_ms)."""
    ms = (ctypes.c_float * 4)()
    st = load_library().prefix_attn_backward_timed(*_backward_args(
        plan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, d_out, lse, dq, dk_prefix, dv_prefix,
        dk_suffix, dv_suffix, workspace, stream), ms)
    if st:
        raise PrefixAttnError(st, "prefix_attn_backward_timed")
    return float(ms[0]), float(ms[1]), float(ms[2]), float(ms[3])


def token_logprob_workspace(num_tokens: int, hidden_dim: int, vocab: int) -> int:
    n = ctypes.c_size_t()
    st = load_library().token_logprob_workspace(int(num_tokens), int(hidden_dim), int(vocab), ctypes.byref(n))
    if st:
        raise PrefixAttnError(st, "token_logprob_workspace")
    return int(n.value)


def token_logprob_forward(hidden, lm_head, targets, logit_scale, logprob_out, lse_out, workspace, stream=None) -> None:
    """token_logprob_forward of the C ABI.  hidden [N,d] / lm_head [V,d] bf16 and targets [N] int32 device tensors;
    logprob_out (and optional lse_out) [N] fp32; workspace uint8 of at least token_logprob_workspace bytes."""
    N, d = int(hidden.shape[0]), int(hidden.shape[1])
    V = int(lm_head.shape[0])
    st = load_library().token_logprob_forward(_ptr(hidden), _ptr(lm_head), _ptr(targets), N, d, V, float(logit_scale),
                                              _ptr(logprob_out), _ptr(lse_out), _ptr(workspace),
                                              _nbytes(workspace, 0), _stream(stream))
    if st:
        raise PrefixAttnError(st, "token_logprob_forward")


def grpo_group_advantages(rewards, advantages_out, stream=None) -> None:
    """grpo_group_advantages of the C ABI.  rewards / advantages_out: [num_groups, group_size] fp32 device tensors."""
    st = load_library().grpo_group_advantages(_ptr(rewards), int(rewards.shape[1]), int(rewards.shape[0]),
                                              _ptr(advantages_out), _stream(stream))
    if st:
        raise PrefixAttnError(st, "grpo_group_advantages")


def prefix_attn_destroy(plan: PrefixAttnPlan) -> None:
    plan.destroy()
