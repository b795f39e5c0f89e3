"""TEST INFRASTRUCTURE - not part of the product.

fp64 CPU oracle for the freeze-aware stage backward, masked AdamW and APF
stability statistics (TimelyFreeze: Sec. 3.2.1 backward decomposition,
App. D.1 mask convention and update rule, Sec. 2.3 APF score).  The arithmetic
lives in ``tf_oracle.c`` (plain C loops); this module only marshals numpy
fp64 arrays into it and holds the tiny host-side selection rule.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the HIP
library's package and the library imports nothing from here.

Parity pins: see the header of ``tf_oracle.c``; no function here is unpinned
against the mathematics, and none can be pinned against paper-printed values
because the paper prints none for these operations.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tf_oracle.c")
# TF_ORACLE_SANITIZE=1 in the environment: the same source built with AddressSanitizer and
# UndefinedBehaviorSanitizer into a library of its own (the process must then have the ASan
# runtime preloaded; tests/test_oracle_sanitized.py runs the pins that way).
_SANITIZE = os.environ.get("TF_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libtf_oracle_san.so" if _SANITIZE else "libtf_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile tf_oracle.c with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = (["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
               if _SANITIZE else ["-O2"])
        cmd = ["gcc"] + opt + ["-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
                               "-std=c11", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dpp = ctypes.POINTER(ctypes.c_void_p)
        lib.oracle_stage_backward.restype = ctypes.c_int
        lib.oracle_stage_backward.argtypes = [
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
            dpp, dpp, dpp, ctypes.c_void_p, dpp, dpp, ctypes.c_int]
        lib.oracle_masked_adamw.restype = ctypes.c_int
        lib.oracle_masked_adamw.argtypes = [
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_double, ctypes.c_double, ctypes.c_double,
            ctypes.c_double, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_double]
        lib.oracle_stability_update.restype = ctypes.c_int
        lib.oracle_stability_update.argtypes = [
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_double, ctypes.c_void_p]
        lib.oracle_score_sums.restype = None
        lib.oracle_score_sums.argtypes = [ctypes.c_int64, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_elem_scores.restype = None
        lib.oracle_elem_scores.argtypes = [ctypes.c_int64, ctypes.c_void_p,
                                           ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_bf16_rne.restype = ctypes.c_double
        lib.oracle_bf16_rne.argtypes = [ctypes.c_double]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a, shape=None, writable=False) -> np.ndarray:
    if not (isinstance(a, np.ndarray) and a.dtype == np.float64 and a.flags.c_contiguous):
        raise TypeError("oracle arrays must be C-contiguous float64 numpy arrays")
    if writable and not a.flags.writeable:
        raise TypeError("output array is read-only")
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"shape {a.shape} != expected {shape}")
    return a


def _ptr_table(arrs):
    tab = (ctypes.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        tab[i] = None if a is None else a.ctypes.data
    return tab


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def stage_backward(shapes: Sequence[tuple], T: int, W, X, dY, freeze_mask,
                   dX, dW, accumulate: bool = False) -> None:
    """dX_l = dY_l W_l^T for every l; dW_l (+)= X_l^T dY_l for l with
    freeze_mask[l] == 0; dW_l of a frozen l is neither read nor written and may
    be None.  All arrays float64, modified in place (Sec. 3.2.1; App. D.1)."""
    L = len(shapes)
    K = np.asarray([s[0] for s in shapes], dtype=np.int64)
    N = np.asarray([s[1] for s in shapes], dtype=np.int64)
    fm = np.ascontiguousarray(np.asarray(freeze_mask, dtype=np.uint8))
    if fm.shape != (L,):
        raise ValueError("freeze_mask must have one byte per layer")
    for l in range(L):
        _f64(W[l], (K[l], N[l]))
        _f64(X[l], (T, K[l]))
        _f64(dY[l], (T, N[l]))
        _f64(dX[l], (T, K[l]), writable=True)
        if not fm[l]:
            _f64(dW[l], (K[l], N[l]), writable=True)
    rc = _load().oracle_stage_backward(
        L, K.ctypes.data, N.ctypes.data, int(T),
        _ptr_table(W), _ptr_table(X), _ptr_table(dY), fm.ctypes.data,
        _ptr_table(dX), _ptr_table([None if fm[l] else dW[l] for l in range(L)]),
        1 if accumulate else 0)
    if rc != 0:
        raise RuntimeError("oracle_stage_backward failed")


def stage_backward_blocks(shapes: Sequence[tuple], T: int, W, X, dY, freeze_mask, row_masks, block_rows: int,
                          dX, dW, accumulate: bool = False) -> None:
    """Stage backward with sub-tensor freezing: as stage_backward, but of an unfrozen
    layer l with row_masks[l] given only the row blocks b with row_masks[l][b] == 0 get
    dW_l[rows of b] (+)= X_l[:, rows of b]^T dY_l; rows of frozen blocks are neither read
    nor written.  dX is always computed in full (Sec. 3.2.1)."""
    L = len(shapes)
    all_frozen = np.ones(L, dtype=np.uint8)
    stage_backward(shapes, T, W, X, dY, all_frozen, dX, [None] * L)              # dX only
    fm = np.asarray(freeze_mask, dtype=np.uint8) if freeze_mask is not None else np.zeros(L, np.uint8)
    for l, (K, N) in enumerate(shapes):
        if fm[l]:
            continue
        rm = None if row_masks is None else row_masks[l]
        if rm is None:
            rm = np.zeros(K // block_rows if K % block_rows == 0 else 1, dtype=np.uint8)
            br = block_rows if K % block_rows == 0 else K
        else:
            br = block_rows
            if K % br or len(rm) != K // br:
                raise ValueError("row mask does not match the layer")
        for b, frozen in enumerate(rm):
            if frozen:
                continue
            rows = slice(b * br, (b + 1) * br)
            Xs = np.ascontiguousarray(X[l][:, rows])
            Ws = np.ascontiguousarray(W[l][rows])
            dWs = np.ascontiguousarray(dW[l][rows])
            scratch = np.zeros((T, br))
            stage_backward([(br, N)], T, [Ws], [Xs], [dY[l]], [0], [scratch], [dWs], accumulate)
            dW[l][rows] = dWs


def stage_backward_shared(shapes: Sequence[tuple], T: int, W, X, dY, freeze_mask, input_group, dX, dW,
                          accumulate: bool = False) -> None:
    """Stage backward in which the layers of one input group share their input: the group's
    input gradient is the sum of its members' dY_l W_l^T (the product with the weights
    concatenated along the output features), written to every member's dX (they may be one
    array).  input_group[l] = -1: a layer of its own.  dW is per layer as in stage_backward."""
    L = len(shapes)
    own = [np.zeros((T, k)) for k, n in shapes]
    stage_backward(shapes, T, W, X, dY, freeze_mask, own, dW, accumulate)
    groups = {}
    for l in range(L):
        g = -1 if input_group is None else int(input_group[l])
        groups.setdefault(g if g >= 0 else -(l + 1), []).append(l)
    for members in groups.values():
        total = np.zeros_like(own[members[0]])
        for l in members:
            total += own[l]
        for l in members:
            dX[l][...] = total


def sample_dx(dY, W, ts, ks) -> np.ndarray:
    """Single elements of the input gradient, one by one: dX[t, k] = sum_n dY[t, n] W[k, n]
    (Sec. 3.2.1, activation-gradient component).  dY [T, N] and W [K, N] may be float32 or
    float64 arrays; every product and sum is done in float64.  For outputs too large to
    compute in full."""
    out = np.empty(len(ts), dtype=np.float64)
    for i, (t, k) in enumerate(zip(ts, ks)):
        out[i] = np.dot(np.asarray(dY[t, :], dtype=np.float64), np.asarray(W[k, :], dtype=np.float64))
    return out


def sample_dw(X, dY, ks, ns) -> np.ndarray:
    """Single elements of the weight gradient: G[k, n] = sum_t X[t, k] dY[t, n]
    (Sec. 3.2.1, parameter-gradient component), in float64."""
    out = np.empty(len(ks), dtype=np.float64)
    for i, (k, n) in enumerate(zip(ks, ns)):
        out[i] = np.dot(np.asarray(X[:, k], dtype=np.float64), np.asarray(dY[:, n], dtype=np.float64))
    return out


def masked_adamw(p, m, v, grad, *, step: int, lr: float, beta1: float, beta2: float,
                 eps: float, weight_decay: float, grad_scale: float = 1.0,
                 p_lowp=None, elem_frozen=None, ema=None, ema_abs=None,
                 ema_decay: float = 0.0) -> None:
    """One tensor's masked AdamW step (+ APF EMAs of the applied update when
    ema/ema_abs are given), in place on flat float64 arrays.  elem_frozen is an
    optional uint8 array, 1 = frozen element, left untouched in every buffer."""
    n = p.size
    for a in (p, m, v):
        _f64(a, writable=True)
    _f64(grad)
    ef = None
    if elem_frozen is not None:
        ef = np.ascontiguousarray(np.asarray(elem_frozen, dtype=np.uint8))
        if ef.size != n:
            raise ValueError("elem_frozen size mismatch")
    for a in (m, v, grad, p_lowp, ema, ema_abs):
        if a is not None and a.size != n:
            raise ValueError("size mismatch")
    rc = _load().oracle_masked_adamw(
        n, p.ctypes.data, m.ctypes.data, v.ctypes.data, grad.ctypes.data,
        float(grad_scale), None if p_lowp is None else _f64(p_lowp, writable=True).ctypes.data,
        None if ef is None else ef.ctypes.data, int(step),
        float(lr), float(beta1), float(beta2), float(eps), float(weight_decay),
        None if ema is None else _f64(ema, writable=True).ctypes.data,
        None if ema_abs is None else _f64(ema_abs, writable=True).ctypes.data,
        float(ema_decay))
    if rc != 0:
        raise ValueError("oracle_masked_adamw rejected its arguments")


def stability_update(delta, ema, ema_abs, ema_decay: float, elem_frozen=None) -> None:
    """E <- aE + (1-a)Delta, A <- aA + (1-a)|Delta| on unfrozen elements (Sec. 2.3)."""
    n = delta.size
    ef = None
    if elem_frozen is not None:
        ef = np.ascontiguousarray(np.asarray(elem_frozen, dtype=np.uint8))
    _load().oracle_stability_update(
        n, _f64(delta).ctypes.data, _f64(ema, writable=True).ctypes.data,
        _f64(ema_abs, writable=True).ctypes.data, float(ema_decay),
        None if ef is None else ef.ctypes.data)


def score_sums(ema, ema_abs) -> tuple:
    """(sum |E|, sum A) over all elements of one tensor."""
    out = np.zeros(2, dtype=np.float64)
    _load().oracle_score_sums(ema.size, _f64(ema).ctypes.data,
                              _f64(ema_abs).ctypes.data, out.ctypes.data)
    return float(out[0]), float(out[1])


def elem_scores(ema, ema_abs) -> np.ndarray:
    """Per-element APF score |E|/E^abs; 1 where E^abs == 0."""
    out = np.empty(ema.size, dtype=np.float64)
    _load().oracle_elem_scores(ema.size, _f64(ema).ctypes.data,
                               _f64(ema_abs).ctypes.data, out.ctypes.data)
    return out.reshape(ema.shape)


def tensor_score(sum_abs_e: float, sum_a: float) -> float:
    """Tensor-level score = (sum |E|) / (sum A); 1 when nothing was ever updated."""
    return 1.0 if sum_a == 0.0 else sum_abs_e / sum_a


def bf16_rne(x: float) -> float:
    return float(_load().oracle_bf16_rne(float(x)))


def n_frozen(r: float, L: int) -> int:
    """Number of frozen tensors for freeze ratio r: ceil(r L), guarded against
    r*L landing a hair above an integer in floating point."""
    return max(0, min(L, int(math.ceil(r * L - 1e-9))))


def select_lowest(scores: Sequence[float], n_freeze: int) -> np.ndarray:
    """Freeze the n_freeze tensors with the lowest score; ties go to the lower
    index.  Returns a uint8 mask, 1 = frozen."""
    L = len(scores)
    if not 0 <= n_freeze <= L:
        raise ValueError("n_freeze out of range")
    order = sorted(range(L), key=lambda i: (float(scores[i]), i))
    mask = np.zeros(L, dtype=np.uint8)
    for i in order[:n_freeze]:
        mask[i] = 1
    return mask


# Metric-aware selection steps around the hot path (plain numpy; see selection.py).
from .selection import (autofreeze_sqnorm, autofreeze_score, autofreeze_select,   # noqa: E402,F401
                        perm32, perm32_inverse, reconcile_mask, pack_bits, unpack_bits,
                        select_row_blocks, row_blocks_to_elem_mask)
