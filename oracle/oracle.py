"""ctypes front end of the CPU oracle (oracle/pac_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.

Everything here is argument marshalling; the arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pac_oracle.c")
# PAC_ORACLE_LIB: a differently built copy of the same source (the sanitizer leg of the CPU tests)
_LIB = os.environ.get("PAC_ORACLE_LIB") or os.path.join(_HERE, "liborc.so")


def build_sanitized(path: str) -> str:
    """The same source built with AddressSanitizer and UndefinedBehaviorSanitizer (host only), for the
    CPU tests' sanitizer leg.  Returns the library path."""
    subprocess.check_call(
        ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=undefined", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
         "-o", path, _SRC, "-lm"])
    return path


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if os.environ.get("PAC_ORACLE_LIB"):
        return _LIB
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i32, i64, dbl = C.c_int32, C.c_int64, C.c_double
        vp = C.c_void_p
        L.orc_num_threads.restype = C.c_int
        L.orc_set_num_threads.argtypes = [C.c_int]
        L.orc_layer_block.restype = i64
        L.orc_layer_block.argtypes = [i32, i32]
        L.orc_param_count.restype = i64
        L.orc_param_count.argtypes = [i32, i32, i32, i32]
        L.orc_f32_to_bf16_bits.restype = C.c_uint16
        L.orc_f32_to_bf16_bits.argtypes = [C.c_float]
        L.orc_bf16_bits_to_f32.restype = C.c_float
        L.orc_bf16_bits_to_f32.argtypes = [C.c_uint16]
        L.orc_cache_elems_per_sample.restype = i64
        L.orc_cache_elems_per_sample.argtypes = [i32, i32, i32]
        L.orc_cache_fill.restype = i64
        L.orc_cache_fill.argtypes = [vp, i32, i32, i32, i32, vp, C.c_int, vp, vp]
        L.orc_bf16_to_f32_array.restype = None
        L.orc_bf16_to_f32_array.argtypes = [vp, i64, vp]
        L.orc_loss_grad.restype = C.c_int
        L.orc_loss_grad.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.orc_adamw.restype = None
        L.orc_adamw.argtypes = [i32, i32, i32, i32, vp, vp, vp, i64, vp, dbl, dbl, dbl, dbl, dbl]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass(frozen=True)
class Dims:
    L: int
    d: int
    r: int
    C: int

    @property
    def layer_block(self) -> int:
        return int(lib().orc_layer_block(self.d, self.r))

    @property
    def P(self) -> int:
        return int(lib().orc_param_count(self.L, self.d, self.r, self.C))


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    lib().orc_set_num_threads(int(n))


def f32_to_bf16_bits(x: float) -> int:
    return int(lib().orc_f32_to_bf16_bits(C.c_float(x)))


def bf16_bits_to_f32(h: int) -> float:
    return float(lib().orc_bf16_bits_to_f32(C.c_uint16(h)))


def cache_elems_per_sample(L: int, length: int, d: int) -> int:
    return int(lib().orc_cache_elems_per_sample(L, length, d))


def cache_fill(acts: np.ndarray, lens=None, as_bf16: bool = True):
    """acts [count][L][n_max][d] fp32 -> (packed cache, off[count]).

    The packed cache is uint16 (bf16 bits) or float32."""
    acts = np.ascontiguousarray(acts, dtype=np.float32)
    count, L, n_max, d = acts.shape
    if lens is None:
        lens_a = np.full(count, n_max, dtype=np.int32)
    else:
        lens_a = np.ascontiguousarray(lens, dtype=np.int32)
        assert lens_a.shape == (count,) and lens_a.min() >= 1 and lens_a.max() <= n_max
    total = int(sum(L * int(x) * d for x in lens_a))
    out = np.empty(total, dtype=np.uint16 if as_bf16 else np.float32)
    off = np.empty(count, dtype=np.int64)
    n = lib().orc_cache_fill(_ptr(acts), count, L, n_max, d, _ptr(lens_a), 1 if as_bf16 else 0,
                             _ptr(out), _ptr(off))
    assert n == total
    return out, off, lens_a


def widen(cache: np.ndarray) -> np.ndarray:
    """Exact float32 view of the stored cache values."""
    if cache.dtype == np.float32:
        return cache
    assert cache.dtype == np.uint16
    out = np.empty(cache.shape, dtype=np.float32)
    lib().orc_bf16_to_f32_array(_ptr(np.ascontiguousarray(cache)), cache.size, _ptr(out))
    return out


def loss_grad(dims: Dims, cache_f32: np.ndarray, off, lens, labels, params,
              want_grads: bool = True):
    """Returns dict(loss, logits[B,C], pooled[B,d], grads[P] or None, glam_abs[L] or None); all float64.

    glam_abs[l] is the sum of the absolute values of the terms whose signed sum is the gradient
    of gate l (its cancellation scale)."""
    cache_f32 = np.ascontiguousarray(cache_f32, dtype=np.float32)
    off = np.ascontiguousarray(off, dtype=np.int64)
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    params = np.ascontiguousarray(params, dtype=np.float64)
    B = int(labels.shape[0])
    assert off.shape == (B,) and lens.shape == (B,)
    assert params.shape == (dims.P,)
    for i in range(B):
        assert 0 <= off[i] and off[i] + dims.L * int(lens[i]) * dims.d <= cache_f32.size
    loss = C.c_double(0.0)
    logits = np.empty((B, dims.C), dtype=np.float64)
    pooled = np.empty((B, dims.d), dtype=np.float64)
    grads = np.empty(dims.P, dtype=np.float64) if want_grads else None
    glam_abs = np.empty(dims.L, dtype=np.float64) if want_grads else None
    rc = lib().orc_loss_grad(dims.L, dims.d, dims.r, dims.C, B, _ptr(cache_f32), _ptr(off),
                             _ptr(lens), _ptr(labels), _ptr(params), C.addressof(loss),
                             _ptr(logits), _ptr(pooled), _ptr(grads), _ptr(glam_abs))
    if rc != 0:
        raise ValueError("oracle rejected the inputs (label/length out of range or no memory)")
    return {"loss": float(loss.value), "logits": logits, "pooled": pooled, "grads": grads, "glam_abs": glam_abs}


@dataclass
class AdamW:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01


def adamw(dims: Dims, p, m, v, t_new: int, g, hp: AdamW) -> None:
    """In-place update of float64 arrays p, m, v; t_new = step count after increment."""
    for a in (p, m, v, g):
        assert a.dtype == np.float64 and a.flags.c_contiguous and a.shape == (dims.P,)
    lib().orc_adamw(dims.L, dims.d, dims.r, dims.C, _ptr(p), _ptr(m), _ptr(v), int(t_new), _ptr(g),
                    hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay)


def step(dims: Dims, cache_f32, off, lens, labels, p, m, v, t: int, hp: AdamW):
    """One training step on float64 state (in place).  Returns (loss, grads, t+1)."""
    out = loss_grad(dims, cache_f32, off, lens, labels, p, want_grads=True)
    adamw(dims, p, m, v, t + 1, out["grads"], hp)
    return out["loss"], out["grads"], t + 1


def param_slices(dims: Dims):
    """Name -> slice of the flat parameter vector (the layout in the C file's header)."""
    d, r, Cc, PL = dims.d, dims.r, dims.C, dims.layer_block
    out = {}
    for l in range(dims.L):
        o = l * PL
        out[f"W_down{l}"] = slice(o, o + d * r)
        out[f"c_down{l}"] = slice(o + d * r, o + d * r + r)
        out[f"W_up{l}"] = slice(o + d * r + r, o + 2 * d * r + r)
        out[f"c_up{l}"] = slice(o + 2 * d * r + r, o + 2 * d * r + r + d)
        out[f"lambda{l}"] = slice(o + 2 * d * r + r + d, o + PL)
    o = dims.L * PL
    out["W_cls"] = slice(o, o + d * Cc)
    out["c_cls"] = slice(o + d * Cc, o + d * Cc + Cc)
    return out
