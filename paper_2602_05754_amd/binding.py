"""ctypes binding of libtf.so.  Argument marshalling only: tensors -> device
pointers, Python lists -> host arrays.  Names and argument order follow
include/tf.h.  torch is used for device memory and streams, nothing else."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

TF_F32 = 0
TF_BF16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtf.so")
_lib = None

EXPORTED_SYMBOLS = [
    "tf_create", "tf_destroy", "tf_strerror", "tf_last_hip_error", "tf_version",
    "tf_stage_backward", "tf_masked_adamw", "tf_stability_update",
    "tf_stability_scores", "tf_select_lowest", "tf_num_frozen",
    "tf_profile_enable", "tf_profile_collect", "tf_assume_lowp_is_rounded_master",
    "tf_autofreeze_norms", "tf_autofreeze_scores", "tf_autofreeze_select", "tf_reconcile_mask",
    "tf_reconcile_mask_static",
    "tf_stage_backward_blocks", "tf_stage_backward_shared", "tf_select_row_blocks", "tf_row_blocks_to_bits",
    "tf_stage_backward_microbatch", "tf_microbatch_plan",
    "tf_pipeline_dag", "tf_dag_start_times", "tf_freeze_ratio_lp", "tf_actual_freeze_ratio",
]

TF_SCHEDULE_GPIPE = 0
TF_SCHEDULE_1F1B = 1
TF_SCHEDULE_INTERLEAVED_1F1B = 2
TF_SCHEDULE_ZBV = 3

KERNEL_KINDS = {0: "dx_mfma", 1: "dw_mfma", 2: "dx_generic", 3: "dw_generic", 4: "adamw", 5: "stability",
                6: "autofreeze", 7: "reconcile"}


class TfError(RuntimeError):
    def __init__(self, code: int, where: str, hip_error: int = 0):
        self.code = code
        self.hip_error = hip_error
        msg = f"{where}: {tf_strerror(code)} (status {code})"
        if hip_error:
            msg += f", hipError_t {hip_error}"
        super().__init__(msg)


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libtf.so, building it first if it has never been built.  Raises if
    it cannot be had: there is no fallback implementation."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, pp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)
    i32, i64, f32, f64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_double
    lib.tf_create.restype = ctypes.c_int
    lib.tf_create.argtypes = [pp, ctypes.c_int]
    lib.tf_destroy.restype = ctypes.c_int
    lib.tf_destroy.argtypes = [vp]
    lib.tf_strerror.restype = ctypes.c_char_p
    lib.tf_strerror.argtypes = [ctypes.c_int]
    lib.tf_last_hip_error.restype = ctypes.c_int
    lib.tf_last_hip_error.argtypes = [vp]
    lib.tf_version.restype = ctypes.c_char_p
    lib.tf_version.argtypes = []
    lib.tf_stage_backward.restype = ctypes.c_int
    lib.tf_stage_backward.argtypes = [vp, vp, i32, vp, i64, ctypes.c_int, vp, vp, vp, vp, vp, vp,
                                      ctypes.c_int, ctypes.c_int]
    lib.tf_stage_backward_microbatch.restype = ctypes.c_int
    lib.tf_stage_backward_microbatch.argtypes = [vp, vp, i32, vp, i64, ctypes.c_int, vp, vp, vp, vp, vp, vp,
                                                 ctypes.c_int, vp]
    lib.tf_masked_adamw.restype = ctypes.c_int
    lib.tf_masked_adamw.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, ctypes.c_int, f32, vp, vp, vp, vp,
                                    f32, f32, f32, f32, f32, vp, vp, f32, vp]
    lib.tf_stability_update.restype = ctypes.c_int
    lib.tf_stability_update.argtypes = [vp, vp, i32, vp, vp, vp, vp, f32, vp, vp, vp]
    lib.tf_stability_scores.restype = ctypes.c_int
    lib.tf_stability_scores.argtypes = [vp, i32, vp]
    lib.tf_select_lowest.restype = ctypes.c_int
    lib.tf_select_lowest.argtypes = [vp, i32, i32, vp]
    lib.tf_microbatch_plan.restype = ctypes.c_int
    lib.tf_microbatch_plan.argtypes = [i32, i32, vp, vp, vp]
    lib.tf_num_frozen.restype = i32
    lib.tf_num_frozen.argtypes = [f64, i32]
    lib.tf_profile_enable.restype = ctypes.c_int
    lib.tf_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.tf_assume_lowp_is_rounded_master.restype = ctypes.c_int
    lib.tf_assume_lowp_is_rounded_master.argtypes = [vp, ctypes.c_int]
    lib.tf_profile_collect.restype = ctypes.c_int
    lib.tf_profile_collect.argtypes = [vp, i32, vp, vp, vp]
    lib.tf_autofreeze_norms.restype = ctypes.c_int
    lib.tf_autofreeze_norms.argtypes = [vp, vp, i32, vp, vp, vp, vp, ctypes.c_int, vp]
    lib.tf_autofreeze_scores.restype = ctypes.c_int
    lib.tf_autofreeze_scores.argtypes = [vp, vp, i32, vp]
    lib.tf_autofreeze_select.restype = ctypes.c_int
    lib.tf_autofreeze_select.argtypes = [vp, i32, i32, f64, vp]
    lib.tf_stage_backward_blocks.restype = ctypes.c_int
    lib.tf_stage_backward_blocks.argtypes = [vp, vp, i32, vp, i64, ctypes.c_int, vp, vp, vp, vp, vp, i32, vp, vp,
                                             ctypes.c_int, ctypes.c_int]
    lib.tf_stage_backward_shared.restype = ctypes.c_int
    lib.tf_stage_backward_shared.argtypes = [vp, vp, i32, vp, i64, ctypes.c_int, vp, vp, vp, vp, vp, i32, vp, vp, vp,
                                             ctypes.c_int, ctypes.c_int]
    lib.tf_select_row_blocks.restype = ctypes.c_int
    lib.tf_select_row_blocks.argtypes = [i32, vp, i32, f64, ctypes.c_uint64, vp, vp]
    lib.tf_row_blocks_to_bits.restype = ctypes.c_int
    lib.tf_row_blocks_to_bits.argtypes = [vp, vp, i32, vp, vp, i32, vp]
    lib.tf_pipeline_dag.restype = ctypes.c_int
    lib.tf_pipeline_dag.argtypes = [i32, i32, ctypes.c_int, i32, vp, vp]
    lib.tf_dag_start_times.restype = ctypes.c_int
    lib.tf_dag_start_times.argtypes = [i32, i32, vp, vp, vp]
    lib.tf_freeze_ratio_lp.restype = ctypes.c_int
    lib.tf_freeze_ratio_lp.argtypes = [i32, i32, ctypes.c_int, vp, vp, f64, f64, vp, vp, vp, vp, vp]
    lib.tf_actual_freeze_ratio.restype = f64
    lib.tf_actual_freeze_ratio.argtypes = [f64, i64, i64, i64]
    lib.tf_reconcile_mask.restype = ctypes.c_int
    lib.tf_reconcile_mask.argtypes = [vp, vp, i32, vp, vp, i64, ctypes.c_uint64, vp]
    lib.tf_reconcile_mask_static.restype = ctypes.c_int
    lib.tf_reconcile_mask_static.argtypes = [vp, vp, i32, vp, vp, i64, ctypes.c_uint64, vp]
    _lib = lib
    return lib


def tf_strerror(code: int) -> str:
    return load_library().tf_strerror(int(code)).decode()


def tf_version() -> str:
    return load_library().tf_version().decode()


# ----------------------------------------------------------------------------
# marshalling helpers
# ----------------------------------------------------------------------------
def _dptr(x) -> Optional[int]:
    """Device pointer of a torch tensor, or a raw int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


_DTYPE_NAME = {TF_F32: "torch.float32", TF_BF16: "torch.bfloat16"}
_DTYPE_CODE = {v: k for k, v in _DTYPE_NAME.items()}


def _device_index(x) -> int:
    """Device index of a tensor on a GPU, -1 for a host tensor."""
    return int(x.device.index or 0) if x.is_cuda else -1


class PtrTable:
    """A list of device buffers marshalled once: the host array of their pointers and their
    sizes in bytes.  Pass it wherever a wrapper takes a list of tensors when the same list is
    handed over call after call (a training loop): the wrapper then checks the sizes with one
    vector comparison and builds nothing.  It holds references to the tensors."""

    def __init__(self, seq):
        self._items = list(seq)
        n = len(self._items)
        self.arr = (ctypes.c_void_p * max(n, 1))()
        self.nbytes = np.full(n, np.iinfo(np.int64).max, dtype=np.int64)     # raw ints: size unknown
        self.dtype_code = np.full(n, -2, dtype=np.int64)                     # -2 unknown (raw int), -1 neither f32 nor bf16
        self.device = np.full(n, -2, dtype=np.int64)                         # -2 unknown, -1 host
        for i, x in enumerate(self._items):
            self.arr[i] = _dptr(x)
            if x is not None and not isinstance(x, int):
                if not x.is_contiguous():
                    raise ValueError(f"entry {i}: tensor must be contiguous")
                self.nbytes[i] = x.numel() * x.element_size()
                self.dtype_code[i] = _DTYPE_CODE.get(str(x.dtype), -1)
                self.device[i] = _device_index(x)
        self.present = np.array([x is not None for x in self._items], dtype=bool)
        self.ptr = ctypes.cast(self.arr, ctypes.c_void_p)

    def __len__(self):
        return len(self._items)

    def __getitem__(self, i):
        return self._items[i]


def _ptr_array(seq, n):
    """Host array of n device pointers (NULL for None); None stays None."""
    if seq is None:
        return None, None
    if len(seq) != n:
        raise ValueError(f"expected {n} entries, got {len(seq)}")
    if isinstance(seq, PtrTable):
        return seq.arr, seq.ptr
    arr = (ctypes.c_void_p * max(n, 1))()
    for i, x in enumerate(seq):
        arr[i] = _dptr(x)
    return arr, ctypes.cast(arr, ctypes.c_void_p)


def _host(arr, dtype, n):
    if arr is None:
        return None, None
    a = np.ascontiguousarray(np.asarray(arr, dtype=dtype))
    if a.size != n:
        raise ValueError(f"expected {n} entries, got {a.size}")
    return a, ctypes.c_void_p(a.ctypes.data)


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


_ELEM_SIZE = {TF_F32: 4, TF_BF16: 2}


def _check_numel(x, numel, dtype_code, what, ctx=None):
    """Host-side guard: a tensor handed to a kernel must hold what the kernel will index, in the
    element type the call names, on the device of the context (raw integers pass unchecked)."""
    if x is None or isinstance(x, int):
        return
    if str(x.dtype) != _DTYPE_NAME[dtype_code]:
        raise ValueError(f"{what}: tensor of {x.dtype} where the call says {_DTYPE_NAME[dtype_code]}")
    if ctx is not None and _device_index(x) != ctx.device_id:
        raise ValueError(f"{what}: tensor on {x.device}, the context is bound to GPU {ctx.device_id}")
    if x.numel() * x.element_size() < numel * _ELEM_SIZE[dtype_code]:
        raise ValueError(f"{what}: buffer of {x.numel() * x.element_size()} bytes is smaller than "
                         f"{numel} elements of {_ELEM_SIZE[dtype_code]} bytes")
    if not x.is_contiguous():
        raise ValueError(f"{what}: tensor must be contiguous")


def _check_seq(seq, numels, dtype_code, what, skip=None, ctx=None):
    """_check_numel over a list of buffers; entries with skip[i] set are not looked at."""
    if seq is None:
        return
    if isinstance(seq, PtrTable):
        need = np.asarray(numels, dtype=np.int64) * _ELEM_SIZE[dtype_code]
        look = seq.present.copy()
        if skip is not None:
            look &= ~np.asarray(skip, dtype=bool)
        bad = look & (seq.nbytes < need)
        if bad.any():
            i = int(np.flatnonzero(bad)[0])
            raise ValueError(f"{what}[{i}]: buffer of {int(seq.nbytes[i])} bytes is smaller than "
                             f"{int(numels[i])} elements of {_ELEM_SIZE[dtype_code]} bytes")
        bad = look & (seq.dtype_code != -2) & (seq.dtype_code != dtype_code)
        if bad.any():
            i = int(np.flatnonzero(bad)[0])
            raise ValueError(f"{what}[{i}]: tensor of {seq[i].dtype} where the call says {_DTYPE_NAME[dtype_code]}")
        if ctx is not None:
            bad = look & (seq.device != -2) & (seq.device != ctx.device_id)
            if bad.any():
                i = int(np.flatnonzero(bad)[0])
                raise ValueError(f"{what}[{i}]: tensor on {seq[i].device}, the context is bound to GPU {ctx.device_id}")
        return
    for i, x in enumerate(seq):
        if skip is not None and skip[i]:
            continue
        _check_numel(x, int(numels[i]), dtype_code, f"{what}[{i}]", ctx)


class Context:
    """Owns a tf_ctx bound to one HIP device."""

    def __init__(self, device_id: int = 0):
        lib = load_library()
        h = ctypes.c_void_p()
        rc = lib.tf_create(ctypes.byref(h), int(device_id))
        if rc != 0:
            raise TfError(rc, "tf_create")
        self._h = h
        self.device_id = device_id

    @property
    def handle(self):
        return self._h

    def last_hip_error(self) -> int:
        return int(load_library().tf_last_hip_error(self._h))

    def profile_enable(self, on: bool = True) -> None:
        rc = load_library().tf_profile_enable(self._h, 1 if on else 0)
        if rc != 0:
            raise TfError(rc, "tf_profile_enable")

    def assume_lowp_is_rounded_master(self, on: bool = True) -> None:
        """tf_assume_lowp_is_rounded_master: see include/tf.h."""
        rc = load_library().tf_assume_lowp_is_rounded_master(self._h, 1 if on else 0)
        if rc != 0:
            raise TfError(rc, "tf_assume_lowp_is_rounded_master")

    def profile_collect(self, capacity: int = 4096):
        """[(kernel kind name, milliseconds)] of the launches since the last collect."""
        kinds = np.zeros(capacity, dtype=np.int32)
        ms = np.zeros(capacity, dtype=np.float32)
        n = ctypes.c_int32(0)
        rc = load_library().tf_profile_collect(self._h, capacity, kinds.ctypes.data, ms.ctypes.data,
                                               ctypes.addressof(n))
        if rc != 0:
            raise TfError(rc, "tf_profile_collect", self.last_hip_error() if rc == -6 else 0)
        return [(KERNEL_KINDS.get(int(k), str(int(k))), float(t)) for k, t in zip(kinds[: n.value], ms[: n.value])]

    def close(self):
        if self._h is not None and self._h.value:
            load_library().tf_destroy(self._h)
        self._h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _raise(ctx, rc, where):
    if rc != 0:
        hip = 0
        if ctx is not None and rc == -6:
            hip = ctx.last_hip_error()
        raise TfError(rc, where, hip)


def _ctx_handle(ctx):
    return None if ctx is None else ctx.handle


# ----------------------------------------------------------------------------
# entry points (same names as the C ABI)
# ----------------------------------------------------------------------------
def tf_stage_backward(ctx, shapes: Sequence[tuple], T: int, io_dtype: int,
                      W, X, dY, freeze_mask, dX, dW, dw_dtype: int,
                      accumulate: bool = False, stream=None) -> None:
    """dX_l = dY_l W_l^T for every layer; dW_l (+)= X_l^T dY_l for layers whose
    freeze_mask entry is 0.  See include/tf.h."""
    lib = load_library()
    L = len(shapes)
    sh = np.ascontiguousarray(np.asarray(shapes, dtype=np.int64).reshape(L, 2))
    fm, fm_p = _host(freeze_mask, np.uint8, L)
    _check_seq(W, sh[:, 0] * sh[:, 1], io_dtype, "W", ctx=ctx)
    _check_seq(dY, T * sh[:, 1], io_dtype, "dY", ctx=ctx)
    _check_seq(dX, T * sh[:, 0], io_dtype, "dX", ctx=ctx)
    _check_seq(X, T * sh[:, 0], io_dtype, "X", fm, ctx=ctx)
    _check_seq(dW, sh[:, 0] * sh[:, 1], dw_dtype, "dW", fm, ctx=ctx)
    kW, pW = _ptr_array(W, L)
    kX, pX = _ptr_array(X, L)
    kdY, pdY = _ptr_array(dY, L)
    kdX, pdX = _ptr_array(dX, L)
    kdW, pdW = _ptr_array(dW, L)
    rc = lib.tf_stage_backward(_ctx_handle(ctx), _stream_handle(stream) if ctx is not None else None,
                               L, sh.ctypes.data, int(T), int(io_dtype),
                               pW, pX, pdY, fm_p, pdX, pdW, int(dw_dtype), 1 if accumulate else 0)
    _raise(ctx, rc, "tf_stage_backward")


def tf_stage_backward_microbatch(ctx, shapes: Sequence[tuple], T: int, io_dtype: int,
                                 W, X, dY, freeze_mask, dX, dW, dw_dtype: int,
                                 accumulate_mask, stream=None) -> None:
    """tf_stage_backward with the choice between dW_l = and dW_l += made layer by layer
    (accumulate_mask[l] = 0 / 1).  See include/tf.h."""
    lib = load_library()
    L = len(shapes)
    sh = np.ascontiguousarray(np.asarray(shapes, dtype=np.int64).reshape(L, 2))
    fm, fm_p = _host(freeze_mask, np.uint8, L)
    am, am_p = _host(accumulate_mask, np.uint8, L)
    _check_seq(W, sh[:, 0] * sh[:, 1], io_dtype, "W", ctx=ctx)
    _check_seq(dY, T * sh[:, 1], io_dtype, "dY", ctx=ctx)
    _check_seq(dX, T * sh[:, 0], io_dtype, "dX", ctx=ctx)
    _check_seq(X, T * sh[:, 0], io_dtype, "X", fm, ctx=ctx)
    _check_seq(dW, sh[:, 0] * sh[:, 1], dw_dtype, "dW", fm, ctx=ctx)
    kW, pW = _ptr_array(W, L)
    kX, pX = _ptr_array(X, L)
    kdY, pdY = _ptr_array(dY, L)
    kdX, pdX = _ptr_array(dX, L)
    kdW, pdW = _ptr_array(dW, L)
    rc = lib.tf_stage_backward_microbatch(_ctx_handle(ctx), _stream_handle(stream) if ctx is not None else None,
                                          L, sh.ctypes.data, int(T), int(io_dtype),
                                          pW, pX, pdY, fm_p, pdX, pdW, int(dw_dtype), am_p)
    _raise(ctx, rc, "tf_stage_backward_microbatch")


def tf_masked_adamw(ctx, numel: Sequence[int], p_master, m, v, grad, grad_dtype: int,
                    step: Sequence[int], lr: float, beta1: float, beta2: float, eps: float,
                    weight_decay: float, grad_scale: float = 1.0, p_lowp=None,
                    tensor_freeze_mask=None, elem_freeze_bits=None,
                    ema=None, ema_abs=None, ema_decay: float = 0.0, score_sums=None,
                    stream=None) -> None:
    """Masked AdamW step, optionally fused with the APF EMAs.  See include/tf.h."""
    lib = load_library()
    n = len(numel)
    ne, ne_p = _host(numel, np.int64, n)
    st, st_p = _host(step, np.int32, n)
    fm, fm_p = _host(tensor_freeze_mask, np.uint8, n)
    for name, seq, dt in (("p", p_master, TF_F32), ("m", m, TF_F32), ("v", v, TF_F32),
                          ("grad", grad, grad_dtype), ("p_lowp", p_lowp, TF_BF16),
                          ("ema", ema, TF_F32), ("ema_abs", ema_abs, TF_F32)):
        _check_seq(seq, ne, dt, name, fm, ctx=ctx)
    for i in range(n if elem_freeze_bits is not None else 0):
        if fm is not None and fm[i]:
            continue
        if elem_freeze_bits[i] is not None and not isinstance(elem_freeze_bits[i], int):
            if elem_freeze_bits[i].numel() * elem_freeze_bits[i].element_size() < 4 * ((int(ne[i]) + 31) // 32):
                raise ValueError(f"elem_freeze_bits[{i}] too small")
    if score_sums is not None and not isinstance(score_sums, int):
        if score_sums.numel() * score_sums.element_size() < 16 * n:
            raise ValueError("score_sums too small")
    keep = [_ptr_array(s, n) for s in (p_master, m, v, grad, p_lowp, elem_freeze_bits, ema, ema_abs)]
    pp = [k[1] for k in keep]
    rc = lib.tf_masked_adamw(_ctx_handle(ctx), _stream_handle(stream) if ctx is not None else None,
                             n, ne_p, pp[0], pp[1], pp[2], pp[3], int(grad_dtype), float(grad_scale),
                             pp[4], fm_p, pp[5], st_p,
                             float(lr), float(beta1), float(beta2), float(eps), float(weight_decay),
                             pp[6], pp[7], float(ema_decay), _dptr(score_sums))
    _raise(ctx, rc, "tf_masked_adamw")


def tf_stability_update(ctx, numel: Sequence[int], delta, ema, ema_abs, ema_decay: float,
                        tensor_freeze_mask=None, elem_freeze_bits=None, score_sums=None,
                        stream=None) -> None:
    """Stand-alone APF EMA update from an explicit fp32 delta.  See include/tf.h."""
    lib = load_library()
    n = len(numel)
    ne, ne_p = _host(numel, np.int64, n)
    fm, fm_p = _host(tensor_freeze_mask, np.uint8, n)
    for i in range(n):
        if fm is not None and fm[i]:
            continue
        for name, seq in (("delta", delta), ("ema", ema), ("ema_abs", ema_abs)):
            if seq is not None:
                _check_numel(seq[i], int(ne[i]), TF_F32, f"{name}[{i}]", ctx)
    keep = [_ptr_array(s, n) for s in (delta, ema, ema_abs, elem_freeze_bits)]
    pp = [k[1] for k in keep]
    rc = lib.tf_stability_update(_ctx_handle(ctx), _stream_handle(stream) if ctx is not None else None,
                                 n, ne_p, pp[0], pp[1], pp[2], float(ema_decay), fm_p, pp[3],
                                 _dptr(score_sums))
    _raise(ctx, rc, "tf_stability_update")


def tf_stability_scores(score_sums_host) -> np.ndarray:
    """Host: per-tensor score = sum|E| / sum A from a host copy of score_sums."""
    lib = load_library()
    s = np.ascontiguousarray(np.asarray(score_sums_host, dtype=np.float64).reshape(-1))
    n = s.size // 2
    out = np.empty(n, dtype=np.float64)
    rc = lib.tf_stability_scores(s.ctypes.data, n, out.ctypes.data)
    _raise(None, rc, "tf_stability_scores")
    return out


def tf_select_lowest(scores, n_freeze: int) -> np.ndarray:
    """Host: uint8 mask, 1 for the n_freeze lowest scores (ties -> lower index)."""
    lib = load_library()
    s = np.ascontiguousarray(np.asarray(scores, dtype=np.float64).reshape(-1))
    out = np.zeros(max(s.size, 1), dtype=np.uint8)
    rc = lib.tf_select_lowest(s.ctypes.data, s.size, int(n_freeze), out.ctypes.data)
    _raise(None, rc, "tf_select_lowest")
    return out[: s.size]


def tf_microbatch_plan(freeze_masks):
    """(accumulate_masks [M x L], step_freeze_mask [L]) of a step whose microbatch m has the freeze
    mask freeze_masks[m].  See include/tf.h."""
    fm = np.ascontiguousarray(np.asarray(freeze_masks, dtype=np.uint8))
    if fm.ndim != 2:
        raise ValueError("freeze_masks: one row per microbatch")
    M, L = fm.shape
    acc = np.zeros((M, L), dtype=np.uint8)
    step = np.zeros(L, dtype=np.uint8)
    rc = load_library().tf_microbatch_plan(M, L, fm.ctypes.data, acc.ctypes.data, step.ctypes.data)
    _raise(None, rc, "tf_microbatch_plan")
    return acc, step


def tf_num_frozen(r: float, n: int) -> int:
    return int(load_library().tf_num_frozen(float(r), int(n)))


def tf_autofreeze_norms(ctx, numel: Sequence[int], p_master, snapshot, sq_norms,
                        tensor_freeze_mask=None, update_snapshot: bool = True, stream=None) -> None:
    """sq_norms[i] = sum((p_master[i] - snapshot[i])^2); snapshot <- p_master on request.  See include/tf.h."""
    lib = load_library()
    n = len(numel)
    ne, ne_p = _host(numel, np.int64, n)
    fm, fm_p = _host(tensor_freeze_mask, np.uint8, n)
    for i in range(n):
        if fm is not None and fm[i]:
            continue
        for name, seq in (("p_master", p_master), ("snapshot", snapshot)):
            if seq is not None:
                _check_numel(seq[i], int(ne[i]), TF_F32, f"{name}[{i}]", ctx)
    keep = [_ptr_array(s, n) for s in (p_master, snapshot)]
    rc = lib.tf_autofreeze_norms(_ctx_handle(ctx), _stream_handle(stream) if ctx is not None else None,
                                 n, ne_p, keep[0][1], keep[1][1], fm_p, int(bool(update_snapshot)), _dptr(sq_norms))
    _raise(ctx, rc, "tf_autofreeze_norms")


def tf_autofreeze_scores(sq_prev, sq_cur) -> np.ndarray:
    """Host: | ||D_prev|| - ||D_cur|| | / ||D_prev|| per layer from squared norms."""
    lib = load_library()
    a = np.ascontiguousarray(np.asarray(sq_prev, dtype=np.float64).reshape(-1))
    b = np.ascontiguousarray(np.asarray(sq_cur, dtype=np.float64).reshape(-1))
    if a.size != b.size:
        raise ValueError("sq_prev and sq_cur differ in length")
    out = np.empty(max(a.size, 1), dtype=np.float64)
    rc = lib.tf_autofreeze_scores(a.ctypes.data, b.ctypes.data, a.size, out.ctypes.data)
    _raise(None, rc, "tf_autofreeze_scores")
    return out[: a.size]


def tf_autofreeze_select(scores, n_already_frozen: int, percentile: float) -> np.ndarray:
    """Host: prefix freezing mask after one stability check (1 = frozen)."""
    lib = load_library()
    s = np.ascontiguousarray(np.asarray(scores, dtype=np.float64).reshape(-1))
    out = np.zeros(max(s.size, 1), dtype=np.uint8)
    rc = lib.tf_autofreeze_select(s.ctypes.data, s.size, int(n_already_frozen), float(percentile), out.ctypes.data)
    _raise(None, rc, "tf_autofreeze_select")
    return out[: s.size]


def tf_reconcile_mask_static(ctx, numel: Sequence[int], elem_bits, n_freeze: int, seed: int, stats=None, stream=None) -> None:
    """tf_reconcile_mask without any allocation (state in a static device array).  See include/tf.h."""
    tf_reconcile_mask(ctx, numel, elem_bits, n_freeze, seed, stats, stream, _entry="tf_reconcile_mask_static")


def tf_reconcile_mask(ctx, numel: Sequence[int], elem_bits, n_freeze: int, seed: int, stats=None, stream=None,
                      _entry: str = "tf_reconcile_mask") -> None:
    """Bring the element masks (device uint32 words, updated in place) to exactly n_freeze ones.  See include/tf.h."""
    lib = load_library()
    n = len(numel)
    ne, ne_p = _host(numel, np.int64, n)
    for i in range(n):
        x = elem_bits[i] if elem_bits is not None else None
        if x is not None and not isinstance(x, int) and x.numel() * x.element_size() < ((int(ne[i]) + 31) // 32) * 4:
            raise ValueError(f"elem_bits[{i}]: buffer smaller than {(int(ne[i]) + 31) // 32} mask words")
    if stats is not None and not isinstance(stats, int) and stats.numel() * stats.element_size() < 24:
        raise ValueError("stats: needs room for 3 int64 values")
    keep = _ptr_array(elem_bits, n)
    rc = getattr(lib, _entry)(_ctx_handle(ctx), _stream_handle(stream) if ctx is not None else None,
                              n, ne_p, keep[1], int(n_freeze), int(seed) & ((1 << 64) - 1), _dptr(stats))
    _raise(ctx, rc, _entry)


def _host_mask_table(row_masks, shapes, block_rows):
    """Host array of host pointers to per-layer uint8 row-block masks (NULL for None)."""
    if row_masks is None:
        return None, None
    L = len(shapes)
    if len(row_masks) != L:
        raise ValueError(f"expected {L} row masks, got {len(row_masks)}")
    keep = []
    arr = (ctypes.c_void_p * max(L, 1))()
    for l, m in enumerate(row_masks):
        if m is None:
            arr[l] = None
            continue
        a = np.ascontiguousarray(np.asarray(m, dtype=np.uint8).reshape(-1))
        K = int(shapes[l][0])
        if block_rows > 0 and K % block_rows == 0 and a.size != K // block_rows:
            raise ValueError(f"row mask {l}: expected {K // block_rows} entries, got {a.size}")
        keep.append(a)
        arr[l] = a.ctypes.data
    return (arr, keep), ctypes.cast(arr, ctypes.c_void_p)


def tf_stage_backward_blocks(ctx, shapes: Sequence[tuple], T: int, io_dtype: int,
                             W, X, dY, freeze_mask, row_block_mask, block_rows: int, dX, dW, dw_dtype: int,
                             accumulate: bool = False, stream=None) -> None:
    """Stage backward with sub-tensor freezing: of an unfrozen layer only the row blocks whose
    row_block_mask entry is 0 get their part of dW.  See include/tf.h."""
    lib = load_library()
    L = len(shapes)
    sh = np.ascontiguousarray(np.asarray(shapes, dtype=np.int64).reshape(L, 2))
    fm, fm_p = _host(freeze_mask, np.uint8, L)
    for l in range(L):
        K, N = int(sh[l, 0]), int(sh[l, 1])
        frozen = fm is not None and fm[l]
        if W is not None: _check_numel(W[l], K * N, io_dtype, f"W[{l}]", ctx)
        if dY is not None: _check_numel(dY[l], T * N, io_dtype, f"dY[{l}]", ctx)
        if dX is not None: _check_numel(dX[l], T * K, io_dtype, f"dX[{l}]", ctx)
        if not frozen:
            if X is not None: _check_numel(X[l], T * K, io_dtype, f"X[{l}]", ctx)
            if dW is not None: _check_numel(dW[l], K * N, dw_dtype, f"dW[{l}]", ctx)
    keep = [_ptr_array(s, L) for s in (W, X, dY, dX, dW)]
    rm_keep, rm_p = _host_mask_table(row_block_mask, [tuple(map(int, r)) for r in sh], int(block_rows))
    rc = lib.tf_stage_backward_blocks(_ctx_handle(ctx), _stream_handle(stream) if ctx is not None else None,
                                      L, sh.ctypes.data, int(T), int(io_dtype),
                                      keep[0][1], keep[1][1], keep[2][1], fm_p, rm_p, int(block_rows),
                                      keep[3][1], keep[4][1], int(dw_dtype), 1 if accumulate else 0)
    _raise(ctx, rc, "tf_stage_backward_blocks")


def tf_stage_backward_shared(ctx, shapes: Sequence[tuple], T: int, io_dtype: int,
                             W, X, dY, freeze_mask, row_block_mask, block_rows: int, input_group, dX, dW, dw_dtype: int,
                             accumulate: bool = False, stream=None) -> None:
    """Stage backward in which layers of one input group share their dX (the sum of the members'
    products).  See include/tf.h."""
    lib = load_library()
    L = len(shapes)
    sh = np.ascontiguousarray(np.asarray(shapes, dtype=np.int64).reshape(L, 2))
    fm, fm_p = _host(freeze_mask, np.uint8, L)
    ig, ig_p = _host(input_group, np.int32, L)
    for l in range(L):
        K, N = int(sh[l, 0]), int(sh[l, 1])
        frozen = fm is not None and fm[l]
        if W is not None: _check_numel(W[l], K * N, io_dtype, f"W[{l}]", ctx)
        if dY is not None: _check_numel(dY[l], T * N, io_dtype, f"dY[{l}]", ctx)
        if dX is not None: _check_numel(dX[l], T * K, io_dtype, f"dX[{l}]", ctx)
        if not frozen:
            if X is not None: _check_numel(X[l], T * K, io_dtype, f"X[{l}]", ctx)
            if dW is not None: _check_numel(dW[l], K * N, dw_dtype, f"dW[{l}]", ctx)
    keep = [_ptr_array(s, L) for s in (W, X, dY, dX, dW)]
    rm_keep, rm_p = _host_mask_table(row_block_mask, [tuple(map(int, r)) for r in sh], int(block_rows))
    rc = lib.tf_stage_backward_shared(_ctx_handle(ctx), _stream_handle(stream) if ctx is not None else None,
                                      L, sh.ctypes.data, int(T), int(io_dtype),
                                      keep[0][1], keep[1][1], keep[2][1], fm_p, rm_p, int(block_rows), ig_p,
                                      keep[3][1], keep[4][1], int(dw_dtype), 1 if accumulate else 0)
    _raise(ctx, rc, "tf_stage_backward_shared")


def tf_select_row_blocks(shapes: Sequence[tuple], block_rows: int, r: float, seed: int):
    """Host: seeded draw of row blocks under a parameter budget.  Returns (list of uint8 masks per layer, frozen params)."""
    lib = load_library()
    L = len(shapes)
    sh = np.ascontiguousarray(np.asarray(shapes, dtype=np.int64).reshape(L, 2))
    counts = [int(k) // int(block_rows) if block_rows > 0 and int(k) % int(block_rows) == 0 else 0 for k, _ in sh]
    flat = np.zeros(max(sum(counts), 1), dtype=np.uint8)
    frozen = ctypes.c_int64(0)
    rc = lib.tf_select_row_blocks(L, sh.ctypes.data, int(block_rows), float(r), int(seed) & ((1 << 64) - 1),
                                  flat.ctypes.data, ctypes.addressof(frozen))
    _raise(None, rc, "tf_select_row_blocks")
    out, o = [], 0
    for c in counts:
        out.append(flat[o:o + c].copy())
        o += c
    return out, int(frozen.value)


def tf_row_blocks_to_bits(ctx, shapes: Sequence[tuple], row_block_mask, block_rows: int, elem_bits, stream=None) -> None:
    """Element masks (device uint32 words, written) of row-block masks.  See include/tf.h."""
    lib = load_library()
    L = len(shapes)
    sh = np.ascontiguousarray(np.asarray(shapes, dtype=np.int64).reshape(L, 2))
    for l in range(L):
        x = elem_bits[l] if elem_bits is not None else None
        words = (int(sh[l, 0]) * int(sh[l, 1]) + 31) // 32
        if x is not None and not isinstance(x, int) and x.numel() * x.element_size() < words * 4:
            raise ValueError(f"elem_bits[{l}]: buffer smaller than {words} mask words")
    keep = _ptr_array(elem_bits, L)
    rm_keep, rm_p = _host_mask_table(row_block_mask, [tuple(map(int, r)) for r in sh], int(block_rows))
    rc = lib.tf_row_blocks_to_bits(_ctx_handle(ctx), _stream_handle(stream) if ctx is not None else None,
                                   L, sh.ctypes.data, rm_p, int(block_rows), keep[1])
    _raise(ctx, rc, "tf_row_blocks_to_bits")


def tf_pipeline_dag(n_stages: int, n_microbatches: int, schedule: int) -> np.ndarray:
    """Host: edges (from, to) of one batch's schedule DAG, an [n_edges x 2] int32 array.  See include/tf.h."""
    lib = load_library()
    n = ctypes.c_int32(0)
    rc = lib.tf_pipeline_dag(int(n_stages), int(n_microbatches), int(schedule), 0, None, ctypes.addressof(n))
    _raise(None, rc, "tf_pipeline_dag")
    edges = np.zeros((max(n.value, 1), 2), dtype=np.int32)
    rc = lib.tf_pipeline_dag(int(n_stages), int(n_microbatches), int(schedule), n.value, edges.ctypes.data, ctypes.addressof(n))
    _raise(None, rc, "tf_pipeline_dag")
    return edges[: n.value]


def tf_dag_start_times(n_nodes: int, edges, w) -> np.ndarray:
    """Host: start times by longest path."""
    lib = load_library()
    e = np.ascontiguousarray(np.asarray(edges, dtype=np.int32).reshape(-1, 2))
    wv = np.ascontiguousarray(np.asarray(w, dtype=np.float64).reshape(-1))
    if wv.size != n_nodes:
        raise ValueError("one duration per node")
    P = np.zeros(max(n_nodes, 1), dtype=np.float64)
    rc = lib.tf_dag_start_times(int(n_nodes), e.shape[0], e.ctypes.data, wv.ctypes.data, P.ctypes.data)
    _raise(None, rc, "tf_dag_start_times")
    return P[:n_nodes]


def tf_freeze_ratio_lp(n_stages: int, n_microbatches: int, schedule: int, w_min, w_max, r_max: float, lam: float) -> dict:
    """Host: expected freeze ratios from measured action times.  See include/tf.h."""
    lib = load_library()
    n_act = 2 * int(n_stages) * int(n_microbatches)
    lo = np.ascontiguousarray(np.asarray(w_min, dtype=np.float64).reshape(-1))
    hi = np.ascontiguousarray(np.asarray(w_max, dtype=np.float64).reshape(-1))
    if lo.size != n_act or hi.size != n_act:
        raise ValueError(f"expected {n_act} durations")
    r = np.zeros(max(n_act, 1)); w = np.zeros(max(n_act, 1)); P = np.zeros(n_act + 2)
    t_max, t_opt = ctypes.c_double(0.0), ctypes.c_double(0.0)
    rc = lib.tf_freeze_ratio_lp(int(n_stages), int(n_microbatches), int(schedule), lo.ctypes.data, hi.ctypes.data,
                                float(r_max), float(lam), r.ctypes.data, w.ctypes.data, P.ctypes.data,
                                ctypes.addressof(t_max), ctypes.addressof(t_opt))
    _raise(None, rc, "tf_freeze_ratio_lp")
    return {"r": r[:n_act], "w": w[:n_act], "P": P, "P_d_max": t_max.value, "P_d": t_opt.value}


def tf_actual_freeze_ratio(r: float, t: int, T_m: int, T_f: int) -> float:
    return float(load_library().tf_actual_freeze_ratio(float(r), int(t), int(T_m), int(T_f)))
