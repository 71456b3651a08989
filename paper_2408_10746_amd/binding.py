"""Thin ctypes binding of libpac.so: the same entry points as include/pac.h.

Argument marshalling only -- every step of the path runs in the library's HIP
kernels.  PyTorch is used by callers for device memory and streams; this module
accepts raw integer addresses (tensor.data_ptr()) and a raw stream handle.
There is no CPU fallback: if the library is missing the import of a symbol fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpac.so")

PAC_OK = 0
PAC_ERR_NULL, PAC_ERR_SHAPE, PAC_ERR_RANGE, PAC_ERR_ALIGN = 1, 2, 3, 4
PAC_ERR_UNSUPPORTED, PAC_ERR_WORKSPACE, PAC_ERR_DEVICE, PAC_ERR_STATE = 5, 6, 7, 8
PAC_BF16, PAC_F32 = 0, 1
PAC_FLAG_PER_LAYER = 1
PAC_FLAG_SPLIT_LAUNCH = 2
PAC_FLAG_LAYER_CHAIN = 4

EXPORTS = [
    "pac_create", "pac_destroy", "pac_status_str", "pac_param_count", "pac_param_offsets",
    "pac_cache_bytes", "pac_workspace_bytes", "pac_step_path", "pac_cache_fill", "pac_cache_lookup",
    "pac_adapter_loss_grad", "pac_adapter_step", "pac_adapter_step_static",
    "pac_probe_hbm_read", "pac_probe_mfma_bf16", "pac_probe_mfma_flops", "pac_probe_hbm_update",
    "pac_profile_begin", "pac_profile_end", "pac_profile_class_name",
    "pac_plan_hybrid", "pac_plan_stage_time",
    "pac_quant_blockwise", "pac_dequant_blockwise", "pac_dequant_linear", "pac_dequant_linear_to_cache",
    "pac_tier_window_bytes", "pac_tier_fill", "pac_tier_stage", "pac_adapter_loss_grad_staged", "pac_adapter_step_staged",
    "pac_ladder_param_count", "pac_ladder_workspace_bytes", "pac_ladder_loss_grad", "pac_ladder_step",
]
PAC_STATIC_WORKSPACE_BYTES = 64 << 20


class pac_config(C.Structure):
    _fields_ = [("L", C.c_int32), ("d", C.c_int32), ("n_max", C.c_int32), ("r", C.c_int32),
                ("C", C.c_int32), ("B_max", C.c_int32), ("N", C.c_int64), ("cache_dtype", C.c_int32),
                ("flags", C.c_int32)]


class pac_adamw(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float)]


class pac_plan_problem(C.Structure):
    _dp = C.POINTER(C.c_double)
    _fields_ = [("L", C.c_int32), ("n_dev", C.c_int32), ("B", C.c_int32), ("M", C.c_int32),
                ("t_f", _dp), ("t_b", _dp), ("mem_fixed", _dp), ("mem_act", _dp), ("mem_budget", _dp),
                ("act_bytes", _dp), ("grad_bytes", _dp), ("train_bytes", _dp), ("bandwidth", C.c_double)]


class pac_plan_result(C.Structure):
    _ip, _dp = C.POINTER(C.c_int32), C.POINTER(C.c_double)
    _fields_ = [("sigma", C.c_int32), ("stage_first_layer", _ip), ("stage_last_layer", _ip),
                ("stage_first_dev", _ip), ("stage_n_dev", _ip), ("samples", _ip), ("slowest_stage", C.c_double),
                ("L_b", C.c_double), ("L_e", C.c_double), ("L_n", C.c_double),
                ("latency_by_stage_count", _dp), ("slowest_by_stage_count", _dp)]


class PacError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_str(status)} (status {status})")


_lib = None


def lib():
    """Load libpac.so (built beforehand by paper_2408_10746_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2408_10746_amd.build`")
        # PyTorch first: it brings its own HIP runtime, and the library must bind to the same one as
        # the device pointers and streams it is handed (loaded the other way round, the system's
        # runtime is loaded as well and launches on PyTorch's streams fail).
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.pac_create.restype = C.c_int
        L.pac_create.argtypes = [C.POINTER(pac_config), C.POINTER(vp)]
        L.pac_destroy.restype = None
        L.pac_destroy.argtypes = [vp]
        L.pac_status_str.restype = C.c_char_p
        L.pac_status_str.argtypes = [C.c_int]
        L.pac_param_count.restype = i64
        L.pac_param_count.argtypes = [vp]
        L.pac_param_offsets.restype = C.c_int
        L.pac_param_offsets.argtypes = [vp, i32, C.POINTER(i64)]
        L.pac_cache_bytes.restype = i64
        L.pac_cache_bytes.argtypes = [vp, vp, i64]
        L.pac_workspace_bytes.restype = i64
        L.pac_workspace_bytes.argtypes = [vp]
        L.pac_step_path.restype = C.c_int32
        L.pac_step_path.argtypes = [vp]
        L.pac_cache_fill.restype = C.c_int
        L.pac_cache_fill.argtypes = [vp, vp, i64, vp, i32, vp, i32, vp, vp]
        L.pac_cache_lookup.restype = C.c_int
        L.pac_cache_lookup.argtypes = [vp, i64, C.POINTER(i64), C.POINTER(i32)]
        L.pac_adapter_loss_grad.restype = C.c_int
        L.pac_adapter_loss_grad.argtypes = [vp, vp, vp, i32, vp, vp, vp, i64, vp, vp, vp, vp]
        L.pac_adapter_step.restype = C.c_int
        L.pac_adapter_step.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, C.POINTER(i64),
                                       C.POINTER(pac_adamw), vp, i64, vp, vp, vp]
        L.pac_adapter_step_static.restype = C.c_int
        L.pac_adapter_step_static.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, C.POINTER(i64),
                                              C.POINTER(pac_adamw), vp, vp, vp]
        L.pac_probe_hbm_read.restype = C.c_int
        L.pac_probe_hbm_read.argtypes = [vp, i64, vp, vp]
        L.pac_probe_mfma_bf16.restype = C.c_int
        L.pac_probe_mfma_bf16.argtypes = [i64, vp, vp]
        L.pac_probe_hbm_update.restype = C.c_int
        L.pac_probe_hbm_update.argtypes = [vp, vp, vp, vp, i64, vp]
        L.pac_probe_mfma_flops.restype = C.c_double
        L.pac_probe_mfma_flops.argtypes = [i64]
        L.pac_tier_window_bytes.restype = i64
        L.pac_tier_window_bytes.argtypes = [vp]
        L.pac_tier_fill.restype = C.c_int
        L.pac_tier_fill.argtypes = [vp, vp, i64, vp, i32, vp, i32, vp, vp, i64, vp]
        L.pac_tier_stage.restype = C.c_int
        L.pac_tier_stage.argtypes = [vp, vp, vp, i32, vp, i64, vp]
        L.pac_adapter_loss_grad_staged.restype = C.c_int
        L.pac_adapter_loss_grad_staged.argtypes = L.pac_adapter_loss_grad.argtypes
        L.pac_adapter_step_staged.restype = C.c_int
        L.pac_adapter_step_staged.argtypes = L.pac_adapter_step.argtypes
        L.pac_quant_blockwise.restype = C.c_int
        L.pac_quant_blockwise.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        L.pac_dequant_blockwise.restype = C.c_int
        L.pac_dequant_blockwise.argtypes = [vp, vp, i64, i32, i32, vp, vp]
        L.pac_dequant_linear.restype = C.c_int
        L.pac_dequant_linear.argtypes = [vp, i32, i32, vp, vp, i32, i32, i32, vp, vp]
        L.pac_dequant_linear_to_cache.restype = C.c_int
        L.pac_dequant_linear_to_cache.argtypes = [vp, vp, i64, vp, i32, vp, i32, vp, i32, vp, vp, i32, i32, vp]
        L.pac_plan_hybrid.restype = C.c_int
        L.pac_plan_hybrid.argtypes = [C.POINTER(pac_plan_problem), C.POINTER(pac_plan_result)]
        L.pac_plan_stage_time.restype = C.c_double
        L.pac_plan_stage_time.argtypes = [C.POINTER(pac_plan_problem), i32, i32, i32, i32, vp]
        L.pac_ladder_param_count.restype = i64
        L.pac_ladder_param_count.argtypes = [vp]
        L.pac_ladder_workspace_bytes.restype = i64
        L.pac_ladder_workspace_bytes.argtypes = [vp, i32]
        L.pac_ladder_loss_grad.restype = C.c_int
        L.pac_ladder_loss_grad.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp, i64, vp, vp, vp, vp]
        L.pac_ladder_step.restype = C.c_int
        L.pac_ladder_step.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp, vp, C.POINTER(i64), C.POINTER(pac_adamw), vp, i64,
                                      vp, vp, vp]
        L.pac_profile_begin.restype = C.c_int
        L.pac_profile_begin.argtypes = [vp]
        L.pac_profile_end.restype = C.c_int
        L.pac_profile_end.argtypes = [vp, i32, C.POINTER(C.c_float), C.POINTER(i32), C.POINTER(i32)]
        L.pac_profile_class_name.restype = C.c_char_p
        L.pac_profile_class_name.argtypes = [i32]
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().pac_status_str(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != PAC_OK:
        raise PacError(status, where)


def _host_i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _host_i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _hp(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ---- the C entry points, one to one ---------------------------------------
def pac_create(L, d, n_max, r, C_, B_max, N, cache_dtype, flags=0) -> int:
    cfg = pac_config(L, d, n_max, r, C_, B_max, N, cache_dtype, flags)
    out = C.c_void_p()
    _check(lib().pac_create(C.byref(cfg), C.byref(out)), "pac_create")
    return out.value


def pac_destroy(ctx) -> None:
    lib().pac_destroy(ctx)


def pac_param_count(ctx) -> int:
    return int(lib().pac_param_count(ctx))


def pac_param_offsets(ctx, layer: int):
    out = (C.c_int64 * 5)()
    _check(lib().pac_param_offsets(ctx, layer, out), "pac_param_offsets")
    return list(out)


def pac_cache_bytes(ctx, lens, count: int) -> int:
    la = _host_i32(lens)
    return int(lib().pac_cache_bytes(ctx, _hp(la), count))


def pac_workspace_bytes(ctx) -> int:
    return int(lib().pac_workspace_bytes(ctx))


def pac_step_path(ctx) -> int:
    return int(lib().pac_step_path(ctx))


def pac_cache_fill(ctx, cache_ptr, cache_bytes, sample_ids, acts_ptr, acts_dtype, lens=None, stream=0) -> None:
    ids = _host_i64(sample_ids)
    la = _host_i32(lens)
    _check(lib().pac_cache_fill(ctx, cache_ptr, cache_bytes, _hp(ids), ids.shape[0], acts_ptr, acts_dtype,
                                _hp(la), stream), "pac_cache_fill")


def pac_cache_lookup(ctx, sample_id: int):
    off, ln = C.c_int64(), C.c_int32()
    _check(lib().pac_cache_lookup(ctx, sample_id, C.byref(off), C.byref(ln)), "pac_cache_lookup")
    return off.value, ln.value


def pac_adapter_loss_grad(ctx, cache_ptr, sample_ids, labels_ptr, params_ptr, ws_ptr, ws_bytes, loss_ptr,
                          logits_ptr=None, grads_ptr=None, stream=0) -> None:
    ids = _host_i64(sample_ids)
    _check(lib().pac_adapter_loss_grad(ctx, cache_ptr, _hp(ids), ids.shape[0], labels_ptr, params_ptr, ws_ptr,
                                       ws_bytes, loss_ptr, logits_ptr, grads_ptr, stream),
           "pac_adapter_loss_grad")


def pac_adapter_step(ctx, cache_ptr, sample_ids, labels_ptr, params_ptr, m_ptr, v_ptr, step: int, hp: pac_adamw,
                     ws_ptr, ws_bytes, loss_ptr, grads_ptr=None, stream=0) -> int:
    """Returns the incremented step count."""
    ids = _host_i64(sample_ids)
    st = C.c_int64(step)
    _check(lib().pac_adapter_step(ctx, cache_ptr, _hp(ids), ids.shape[0], labels_ptr, params_ptr, m_ptr, v_ptr,
                                  C.byref(st), C.byref(hp), ws_ptr, ws_bytes, loss_ptr, grads_ptr, stream),
           "pac_adapter_step")
    return st.value


def pac_adapter_step_static(ctx, cache_ptr, sample_ids, labels_ptr, params_ptr, m_ptr, v_ptr, step: int,
                            hp: pac_adamw, loss_ptr, grads_ptr=None, stream=0) -> int:
    """pac_adapter_step on the library's own static workspace.  Returns the incremented step count."""
    ids = _host_i64(sample_ids)
    st = C.c_int64(step)
    _check(lib().pac_adapter_step_static(ctx, cache_ptr, _hp(ids), ids.shape[0], labels_ptr, params_ptr, m_ptr,
                                         v_ptr, C.byref(st), C.byref(hp), loss_ptr, grads_ptr, stream),
           "pac_adapter_step_static")
    return st.value


def pac_probe_hbm_read(buf_ptr, nbytes: int, sink_ptr, stream=0) -> None:
    _check(lib().pac_probe_hbm_read(buf_ptr, nbytes, sink_ptr, stream), "pac_probe_hbm_read")


def pac_probe_mfma_bf16(iters: int, sink_ptr, stream=0) -> None:
    _check(lib().pac_probe_mfma_bf16(iters, sink_ptr, stream), "pac_probe_mfma_bf16")


def pac_probe_hbm_update(p_ptr, m_ptr, v_ptr, g_ptr, n: int, stream=0) -> None:
    _check(lib().pac_probe_hbm_update(p_ptr, m_ptr, v_ptr, g_ptr, n, stream), "pac_probe_hbm_update")


def pac_probe_mfma_flops(iters: int) -> float:
    return float(lib().pac_probe_mfma_flops(iters))


def _plan_problem(t_f, t_b, mem_fixed, mem_act, mem_budget, act_bytes, grad_bytes, train_bytes, bandwidth, M):
    """Marshals numpy arrays into a pac_plan_problem; returns (struct, arrays kept alive)."""
    arrs = [np.ascontiguousarray(a, dtype=np.float64) for a in
            (t_f, t_b, mem_fixed, mem_act, mem_budget, act_bytes, grad_bytes, train_bytes)]
    n_dev, L, B1 = arrs[0].shape
    dp = C.POINTER(C.c_double)
    prob = pac_plan_problem(L, n_dev, B1 - 1, int(M), *[a.ctypes.data_as(dp) for a in arrs], float(bandwidth))
    return prob, arrs


def pac_plan_hybrid(t_f, t_b, mem_fixed, mem_act, mem_budget, act_bytes, grad_bytes, train_bytes, bandwidth, M) -> dict:
    """Algorithm 1 of Sec. 5.1 on host arrays (t_f, t_b: [n_dev][L][B+1]).  Returns the chosen configuration."""
    prob, keep = _plan_problem(t_f, t_b, mem_fixed, mem_act, mem_budget, act_bytes, grad_bytes, train_bytes, bandwidth, M)
    S = min(prob.L, prob.n_dev)
    ia = [np.zeros(S, dtype=np.int32) for _ in range(4)]
    samples = np.zeros(prob.n_dev, dtype=np.int32)
    lat, slow = np.zeros(S + 1), np.zeros(S + 1)
    ip, dp = C.POINTER(C.c_int32), C.POINTER(C.c_double)
    res = pac_plan_result(0, *[a.ctypes.data_as(ip) for a in ia], samples.ctypes.data_as(ip), 0.0, 0.0, 0.0, 0.0,
                          lat.ctypes.data_as(dp), slow.ctypes.data_as(dp))
    _check(lib().pac_plan_hybrid(C.byref(prob), C.byref(res)), "pac_plan_hybrid")
    s = res.sigma
    return {"sigma": s, "stage_first_layer": ia[0][:s].tolist(), "stage_last_layer": ia[1][:s].tolist(),
            "stage_first_dev": ia[2][:s].tolist(), "stage_n_dev": ia[3][:s].tolist(), "samples": samples.tolist(),
            "slowest_stage": res.slowest_stage, "L_b": res.L_b, "L_e": res.L_e, "L_n": res.L_n,
            "latency_by_stage_count": lat, "slowest_by_stage_count": slow}


def pac_plan_stage_time(t_f, t_b, mem_fixed, mem_act, mem_budget, x, y, d_first, n):
    """T(x -> y, {d_first ..}) of Eq. "dp2" and the dispatch that attains it."""
    L = np.asarray(t_f).shape[1]
    z = np.zeros(L)
    prob, keep = _plan_problem(t_f, t_b, mem_fixed, mem_act, mem_budget, z, z, z, 1.0, 1)
    samples = np.zeros(max(n, 1), dtype=np.int32)
    t = lib().pac_plan_stage_time(C.byref(prob), x, y, d_first, n, samples.ctypes.data_as(C.c_void_p))
    return float(t), samples.tolist()


def pac_tier_window_bytes(ctx) -> int:
    return int(lib().pac_tier_window_bytes(ctx))


def pac_tier_fill(ctx, host_ptr, host_bytes, sample_ids, acts_ptr, acts_dtype, lens, window_ptr, window_bytes, stream=0) -> None:
    ids = _host_i64(sample_ids)
    la = _host_i32(lens)
    _check(lib().pac_tier_fill(ctx, host_ptr, host_bytes, _hp(ids), ids.shape[0], acts_ptr, acts_dtype, _hp(la), window_ptr,
                               window_bytes, stream), "pac_tier_fill")


def pac_tier_stage(ctx, host_ptr, sample_ids, window_ptr, window_bytes, stream=0) -> None:
    ids = _host_i64(sample_ids)
    _check(lib().pac_tier_stage(ctx, host_ptr, _hp(ids), ids.shape[0], window_ptr, window_bytes, stream), "pac_tier_stage")


def pac_adapter_loss_grad_staged(ctx, window_ptr, sample_ids, labels_ptr, params_ptr, ws_ptr, ws_bytes, loss_ptr,
                                 logits_ptr=None, grads_ptr=None, stream=0) -> None:
    ids = _host_i64(sample_ids)
    _check(lib().pac_adapter_loss_grad_staged(ctx, window_ptr, _hp(ids), ids.shape[0], labels_ptr, params_ptr, ws_ptr,
                                              ws_bytes, loss_ptr, logits_ptr, grads_ptr, stream),
           "pac_adapter_loss_grad_staged")


def pac_adapter_step_staged(ctx, window_ptr, sample_ids, labels_ptr, params_ptr, m_ptr, v_ptr, step: int, hp: pac_adamw,
                            ws_ptr, ws_bytes, loss_ptr, grads_ptr=None, stream=0) -> int:
    ids = _host_i64(sample_ids)
    st = C.c_int64(step)
    _check(lib().pac_adapter_step_staged(ctx, window_ptr, _hp(ids), ids.shape[0], labels_ptr, params_ptr, m_ptr, v_ptr,
                                         C.byref(st), C.byref(hp), ws_ptr, ws_bytes, loss_ptr, grads_ptr, stream),
           "pac_adapter_step_staged")
    return st.value


def pac_quant_blockwise(x_ptr, n: int, block: int, bits: int, codes_ptr, consts_ptr, stream=0) -> None:
    _check(lib().pac_quant_blockwise(x_ptr, n, block, bits, codes_ptr, consts_ptr, stream), "pac_quant_blockwise")


def pac_dequant_blockwise(codes_ptr, consts_ptr, n: int, block: int, bits: int, out_ptr, stream=0) -> None:
    _check(lib().pac_dequant_blockwise(codes_ptr, consts_ptr, n, block, bits, out_ptr, stream), "pac_dequant_blockwise")


def pac_dequant_linear(x_ptr, M: int, K: int, codes_ptr, consts_ptr, N: int, block: int, bits: int, y_ptr, stream=0) -> None:
    _check(lib().pac_dequant_linear(x_ptr, M, K, codes_ptr, consts_ptr, N, block, bits, y_ptr, stream), "pac_dequant_linear")


def pac_dequant_linear_to_cache(ctx, cache_ptr, cache_bytes, sample_ids, lens, layer: int, x_ptr, K: int, codes_ptr,
                                consts_ptr, block: int, bits: int, stream=0) -> None:
    ids = _host_i64(sample_ids)
    la = _host_i32(lens)
    _check(lib().pac_dequant_linear_to_cache(ctx, cache_ptr, cache_bytes, _hp(ids), ids.shape[0], _hp(la), layer, x_ptr, K,
                                             codes_ptr, consts_ptr, block, bits, stream), "pac_dequant_linear_to_cache")


def pac_profile_begin(ctx) -> None:
    _check(lib().pac_profile_begin(ctx), "pac_profile_begin")


def pac_profile_end(ctx):
    """Returns {class name: (total ms, launches)} for the classes that ran."""
    n = 128
    ms = (C.c_float * n)()
    launches = (C.c_int32 * n)()
    k = C.c_int32(0)
    _check(lib().pac_profile_end(ctx, n, ms, launches, C.byref(k)), "pac_profile_end")
    out = {}
    for i in range(k.value):
        if launches[i]:
            out[lib().pac_profile_class_name(i).decode()] = (float(ms[i]), int(launches[i]))
    return out


def pac_ladder_param_count(ctx) -> int:
    return int(lib().pac_ladder_param_count(ctx))


def pac_ladder_workspace_bytes(ctx, heads: int) -> int:
    return int(lib().pac_ladder_workspace_bytes(ctx, heads))


def pac_ladder_loss_grad(ctx, cache_ptr, sample_ids, labels_ptr, heads, params_ptr, ws_ptr, ws_bytes, loss_ptr,
                         logits_ptr=None, grads_ptr=None, stream=0) -> None:
    ids = _host_i64(sample_ids)
    _check(lib().pac_ladder_loss_grad(ctx, cache_ptr, _hp(ids), ids.shape[0], labels_ptr, heads, params_ptr, ws_ptr,
                                      ws_bytes, loss_ptr, logits_ptr, grads_ptr, stream), "pac_ladder_loss_grad")


def pac_ladder_step(ctx, cache_ptr, sample_ids, labels_ptr, heads, params_ptr, m_ptr, v_ptr, step: int, hp: pac_adamw,
                    ws_ptr, ws_bytes, loss_ptr, grads_ptr=None, stream=0) -> int:
    ids = _host_i64(sample_ids)
    st = C.c_int64(step)
    _check(lib().pac_ladder_step(ctx, cache_ptr, _hp(ids), ids.shape[0], labels_ptr, heads, params_ptr, m_ptr, v_ptr,
                                 C.byref(st), C.byref(hp), ws_ptr, ws_bytes, loss_ptr, grads_ptr, stream),
           "pac_ladder_step")
    return st.value
