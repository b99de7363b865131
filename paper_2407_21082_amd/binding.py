"""ctypes binding of libeh (see include/eh.h).  Argument marshalling only: every
step of the method runs inside the library's HIP kernels.  PyTorch supplies
device memory (``tensor.data_ptr()``) and the current stream, nothing else.

There is no CPU or eager fallback: if libeh.so is missing, stale or fails to
load, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch  # noqa: F401  (loaded first so that libeh binds to the same HIP runtime)

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libeh.so")

EH_OK = 0
EH_F32, EH_BF16 = 0, 1
STATUS_NAMES = {0: "EH_OK", 1: "EH_ERR_NULL", 2: "EH_ERR_SHAPE", 3: "EH_ERR_DTYPE",
                4: "EH_ERR_RANGE", 5: "EH_ERR_HIP", 6: "EH_ERR_WORKSPACE"}

# every symbol include/eh.h declares
EXPORTS = ["eh_create", "eh_destroy", "eh_eval", "eh_eval_noalloc", "eh_eval_heads", "eh_eval_heads_metrics", "eh_exit_decide", "eh_cascade", "dssd_verify", "dssd_draft", "dssd_tally", "eh_head_losses",
           "eh_calibrate", "eh_check", "eh_set_spin_limit", "eh_last_error", "eh_version"]
# the measurement entry points include/eh_probe.h declares
PROBE_EXPORTS = ["eh_probe_read_weights", "eh_probe_mfma", "eh_probe_calibrate_sorted"]


class EhError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


class _Config(C.Structure):
    _fields_ = [
        ("d", C.c_int32), ("V", C.c_int32), ("n_heads", C.c_int32), ("max_rows", C.c_int32),
        ("w_dtype", C.c_int32), ("h_dtype", C.c_int32), ("ln_eps", C.c_float), ("device", C.c_int32),
        ("W", C.POINTER(C.c_void_p)), ("gamma", C.POINTER(C.c_void_p)), ("beta", C.POINTER(C.c_void_p)),
        ("bias", C.POINTER(C.c_void_p)), ("tau", C.POINTER(C.c_float)),
    ]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} not found: build it with `python -m paper_2407_21082_amd.build` "
            "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.eh_create.argtypes = [C.POINTER(_Config), C.POINTER(vp)]
    lib.eh_destroy.argtypes = [vp]
    lib.eh_eval.argtypes = [vp, i32, vp, i64, vp, vp, i32, vp, vp, vp, vp]
    lib.eh_eval_noalloc.argtypes = [vp, i32, vp, i64, vp, vp, i32, vp, vp, vp, vp]
    lib.eh_eval_heads.argtypes = [vp, i32, i32, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.eh_eval_heads_metrics.argtypes = [vp, i32, i32, vp, i64, i64, i32, vp, vp, vp, vp, vp, vp]
    lib.eh_exit_decide.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.eh_cascade.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp, vp, vp]
    lib.dssd_verify.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.dssd_draft.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.dssd_tally.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
    lib.eh_head_losses.argtypes = [vp, i32, vp, i64, vp, i64, vp, i32, C.c_float, vp, vp, vp, vp]
    lib.eh_calibrate.argtypes = [vp, vp, vp, vp, i64, C.POINTER(C.c_double), i32, vp, vp, vp]
    lib.eh_check.argtypes = [vp, vp]
    lib.eh_set_spin_limit.argtypes = [vp, i32]
    lib.eh_probe_read_weights.argtypes = [vp, i32, i32, i32, i32, vp, C.POINTER(i64), vp]
    lib.eh_probe_mfma.argtypes = [vp, i32, i32, vp, C.POINTER(C.c_double), vp]
    lib.eh_probe_read_weights.restype = C.c_int
    lib.eh_probe_mfma.restype = C.c_int
    lib.eh_last_error.argtypes = [vp]
    lib.eh_last_error.restype = C.c_char_p
    lib.eh_version.argtypes = []
    lib.eh_version.restype = C.c_char_p
    for name in ("eh_create", "eh_destroy", "eh_eval", "eh_eval_noalloc", "eh_eval_heads", "eh_eval_heads_metrics", "eh_exit_decide", "eh_cascade",
                 "dssd_verify", "dssd_draft", "dssd_tally", "eh_head_losses", "eh_calibrate", "eh_check", "eh_set_spin_limit"):
        getattr(lib, name).restype = C.c_int
    return lib


lib = _load()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _check(status: int, handle) -> None:
    if status != EH_OK:
        raise EhError(status, lib.eh_last_error(handle).decode())


def eh_version() -> str:
    return lib.eh_version().decode()


class EhContext:
    """Owner of an ``eh_ctx*``; freed by ``eh_destroy`` or on garbage collection."""

    def __init__(self, handle: int, d: int, V: int, n_heads: int, max_rows: int, dtype: torch.dtype,
                 device: torch.device):
        self.handle = C.c_void_p(handle)
        self.d, self.V, self.n_heads, self.max_rows = d, V, n_heads, max_rows
        self.dtype, self.device = dtype, device

    def __del__(self):
        try:
            eh_destroy(self)
        except Exception:
            pass


def eh_create(W: Sequence[torch.Tensor], gamma: Sequence[torch.Tensor], beta: Sequence[torch.Tensor],
              tau: Sequence[float], max_rows: int, ln_eps: float = 1e-5,
              bias: Optional[Sequence[torch.Tensor]] = None) -> EhContext:
    n = len(W)
    V, d = W[0].shape
    dt = W[0].dtype
    code = {torch.float32: EH_F32, torch.bfloat16: EH_BF16}.get(dt)
    if code is None:
        raise EhError(3, f"unsupported dtype {dt}")
    dev = W[0].device
    for l in range(n):
        assert W[l].is_cuda and W[l].is_contiguous() and W[l].shape == (V, d) and W[l].dtype == dt
        assert gamma[l].dtype == torch.float32 and gamma[l].is_contiguous() and gamma[l].numel() == d
        assert beta[l].dtype == torch.float32 and beta[l].is_contiguous() and beta[l].numel() == d
    arr = C.c_void_p * n
    cfg = _Config(d=d, V=V, n_heads=n, max_rows=max_rows, w_dtype=code, h_dtype=code, ln_eps=ln_eps,
                  device=dev.index or 0,
                  W=arr(*[w.data_ptr() for w in W]),
                  gamma=arr(*[g.data_ptr() for g in gamma]),
                  beta=arr(*[b.data_ptr() for b in beta]),
                  bias=arr(*[b.data_ptr() for b in bias]) if bias is not None else None,
                  tau=(C.c_float * n)(*[float(t) for t in tau]))
    torch.cuda.synchronize(dev)       # the library copies the weights synchronously
    out = C.c_void_p()
    st = lib.eh_create(C.byref(cfg), C.byref(out))
    if st != EH_OK:
        raise EhError(st, lib.eh_last_error(None).decode())
    return EhContext(out.value, d, V, n, max_rows, dt, dev)


def eh_destroy(ctx: EhContext) -> None:
    if ctx.handle:
        lib.eh_destroy(ctx.handle)
        ctx.handle = C.c_void_p(None)


def eh_eval(ctx: EhContext, head: int, h: torch.Tensor, n_rows: int, H: Optional[torch.Tensor],
            lse: Optional[torch.Tensor], argmax: Optional[torch.Tensor],
            row_idx: Optional[torch.Tensor] = None, n_rows_dev: Optional[torch.Tensor] = None,
            row_stride: Optional[int] = None, stream=None) -> None:
    stride = h.stride(-2) if row_stride is None and h.dim() >= 2 else (row_stride or ctx.d)
    _check(lib.eh_eval(ctx.handle, head, _ptr(h), stride, _ptr(row_idx), _ptr(n_rows_dev), n_rows,
                       _ptr(H), _ptr(lse), _ptr(argmax), _stream(stream)), ctx.handle)


def eh_eval_noalloc(ctx: EhContext, head: int, h: torch.Tensor, n_rows: int, H: Optional[torch.Tensor],
                    lse: Optional[torch.Tensor], argmax: Optional[torch.Tensor],
                    row_idx: Optional[torch.Tensor] = None, n_rows_dev: Optional[torch.Tensor] = None,
                    row_stride: Optional[int] = None, stream=None) -> None:
    """eh_eval on the library's static workspace (no allocation of any kind in the call)."""
    stride = h.stride(-2) if row_stride is None and h.dim() >= 2 else (row_stride or ctx.d)
    _check(lib.eh_eval_noalloc(ctx.handle, head, _ptr(h), stride, _ptr(row_idx), _ptr(n_rows_dev), n_rows,
                               _ptr(H), _ptr(lse), _ptr(argmax), _stream(stream)), ctx.handle)


def eh_eval_heads(ctx: EhContext, head0: int, n_heads_eval: int, h_layers: torch.Tensor, n_rows: int,
                  H: Optional[torch.Tensor], lse: Optional[torch.Tensor], argmax: Optional[torch.Tensor],
                  stream=None) -> None:
    """h_layers: [n_heads_eval, n_rows, d] (any strides on the first two axes); outputs
    [n_heads_eval, n_rows] contiguous."""
    _check(lib.eh_eval_heads(ctx.handle, head0, n_heads_eval, _ptr(h_layers), h_layers.stride(0),
                             h_layers.stride(1), n_rows, _ptr(H), _ptr(lse), _ptr(argmax),
                             _stream(stream)), ctx.handle)


def eh_eval_heads_metrics(ctx: EhContext, head0: int, n_heads_eval: int, h_layers: torch.Tensor, n_rows: int,
                          H: Optional[torch.Tensor], lse: Optional[torch.Tensor],
                          argmax: Optional[torch.Tensor], max_prob: Optional[torch.Tensor],
                          margin: Optional[torch.Tensor], stream=None) -> None:
    """eh_eval_heads plus max_prob and margin, each [n_heads_eval, n_rows] float32 or None."""
    _check(lib.eh_eval_heads_metrics(ctx.handle, head0, n_heads_eval, _ptr(h_layers), h_layers.stride(0),
                                     h_layers.stride(1), n_rows, _ptr(H), _ptr(lse), _ptr(argmax),
                                     _ptr(max_prob), _ptr(margin), _stream(stream)), ctx.handle)


def eh_exit_decide(ctx: EhContext, head: int, H: torch.Tensor, argmax: torch.Tensor, n_rows: int,
                   exit_layer: torch.Tensor, token: torch.Tensor, active_idx_out: torch.Tensor,
                   n_active_out: torch.Tensor, row_idx: Optional[torch.Tensor] = None,
                   n_rows_dev: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(lib.eh_exit_decide(ctx.handle, head, _ptr(H), _ptr(argmax), _ptr(row_idx), _ptr(n_rows_dev),
                              n_rows, _ptr(exit_layer), _ptr(token), _ptr(active_idx_out),
                              _ptr(n_active_out), _stream(stream)), ctx.handle)


def eh_cascade(ctx: EhContext, h_layers: torch.Tensor, n_rows: int, exit_layer: torch.Tensor,
               token: torch.Tensor, H_out: Optional[torch.Tensor] = None,
               n_evals_out: Optional[torch.Tensor] = None, stream=None) -> None:
    """h_layers: [n_heads, n_rows, d] (any strides on the first two axes)."""
    _check(lib.eh_cascade(ctx.handle, _ptr(h_layers), h_layers.stride(0), h_layers.stride(1), n_rows,
                          _ptr(exit_layer), _ptr(token), _ptr(H_out), _ptr(n_evals_out),
                          _stream(stream)), ctx.handle)


DRAFT_REASONS = {0: "limit", 1: "eos", 2: "fallback", 3: "exhausted"}


def dssd_draft(ctx: EhContext, h_positions: torch.Tensor, limit: int, eos_token: int, draft: torch.Tensor,
               draft_len: torch.Tensor, exit_layers: torch.Tensor, stop_reason: Optional[torch.Tensor] = None,
               fallback_token: Optional[torch.Tensor] = None, n_evals_out: Optional[torch.Tensor] = None,
               stream=None) -> None:
    """h_positions: [n_positions, n_heads, d] (any strides on the first two axes)."""
    _check(lib.dssd_draft(ctx.handle, _ptr(h_positions), h_positions.stride(0), h_positions.stride(1),
                          h_positions.shape[0], limit, eos_token, _ptr(draft), _ptr(draft_len), _ptr(exit_layers),
                          _ptr(stop_reason), _ptr(fallback_token), _ptr(n_evals_out), _stream(stream)), ctx.handle)


def dssd_tally(ctx: EhContext, draft_len: Optional[torch.Tensor], accepted: torch.Tensor, B: int, k: int,
               exit_layers: Optional[torch.Tensor], counters: torch.Tensor, stream=None) -> None:
    """counters: int64[5] on the device = rounds, drafted, accepted, wasted, exit-layer sum (accumulated)."""
    _check(lib.dssd_tally(ctx.handle, _ptr(draft_len), _ptr(accepted), B, k, _ptr(exit_layers), _ptr(counters),
                          _stream(stream)), ctx.handle)


def eh_head_losses(ctx: EhContext, head: int, h_head: torch.Tensor, h_model: torch.Tensor,
                   labels: Optional[torch.Tensor], n_rows: int, alpha: float, kl: Optional[torch.Tensor],
                   ce: Optional[torch.Tensor], loss: torch.Tensor, stream=None) -> None:
    """h_head, h_model: [n_rows, d] (row stride free); loss: float[3] = L_CE, L_KL, L_hyb."""
    _check(lib.eh_head_losses(ctx.handle, head, _ptr(h_head), h_head.stride(0), _ptr(h_model), h_model.stride(0),
                              _ptr(labels), n_rows, alpha, _ptr(kl), _ptr(ce), _ptr(loss), _stream(stream)),
           ctx.handle)


def eh_calibrate(ctx: EhContext, H: torch.Tensor, pred: torch.Tensor, ref: torch.Tensor, eps,
                 tau_out: torch.Tensor, n_exit_out: Optional[torch.Tensor] = None, stream=None) -> None:
    """H, pred, ref: device [M]; eps: sequence of floats in [0, 1]; tau_out: device [len(eps)] float32;
    n_exit_out: device [len(eps)] int64 or None."""
    arr = (C.c_double * len(eps))(*[float(e) for e in eps])
    _check(lib.eh_calibrate(ctx.handle, _ptr(H), _ptr(pred), _ptr(ref), H.numel(), arr, len(eps),
                            _ptr(tau_out), _ptr(n_exit_out), _stream(stream)), ctx.handle)


def eh_check(ctx: EhContext, stream=None) -> None:
    """Synchronise the stream and raise if a kernel reported a device-side failure."""
    _check(lib.eh_check(ctx.handle, _stream(stream)), ctx.handle)


def eh_set_spin_limit(ctx: EhContext, polls: int) -> None:
    """Bound of the persistent kernel's waits for other workgroups (polls before it gives up)."""
    _check(lib.eh_set_spin_limit(ctx.handle, polls), ctx.handle)


PROBE_READ_REGISTERS, PROBE_READ_LDS = 0, 1


def eh_probe_read_weights(ctx: EhContext, how: int, per_head: bool, head0: int, n_heads_read: int,
                          sink: torch.Tensor, stream=None) -> int:
    """Plain read of the context's weights (measurement only); returns the bytes one call reads."""
    n = C.c_int64(0)
    _check(lib.eh_probe_read_weights(ctx.handle, how, 1 if per_head else 0, head0, n_heads_read, _ptr(sink),
                                     C.byref(n), _stream(stream)), ctx.handle)
    return n.value


def eh_probe_mfma(ctx: EhContext, iters: int, random_operands: bool, sink: torch.Tensor, stream=None) -> float:
    """Registers-only matrix instruction stream (measurement only); returns the flops of one call."""
    f = C.c_double(0.0)
    _check(lib.eh_probe_mfma(ctx.handle, iters, 1 if random_operands else 0, _ptr(sink), C.byref(f),
                             _stream(stream)), ctx.handle)
    return f.value


def eh_probe_calibrate_sorted(ctx: EhContext) -> int:
    """How many eh_calibrate calls on this context the full sort had to serve."""
    n = C.c_int64(0)
    _check(lib.eh_probe_calibrate_sorted(ctx.handle, C.byref(n)), ctx.handle)
    return n.value


def dssd_verify(ctx: EhContext, f_final: torch.Tensor, draft: torch.Tensor,
                draft_len: Optional[torch.Tensor], accepted: torch.Tensor, next_token: torch.Tensor,
                target: Optional[torch.Tensor] = None, stream=None) -> None:
    B, k1, _ = f_final.shape
    assert f_final.is_contiguous()
    _check(lib.dssd_verify(ctx.handle, _ptr(f_final), _ptr(draft), _ptr(draft_len), B, k1 - 1,
                           _ptr(accepted), _ptr(next_token), _ptr(target), _stream(stream)), ctx.handle)
