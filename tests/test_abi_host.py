"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2408_10746_amd import binding as pb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not h.endswith(".h"):
            continue
        src = open(os.path.join(ROOT, "include", h)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(pac_[a-z0-9_]+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert len(names) >= 11
    lib = pb.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/pac.h but not exported"
    assert sorted(pb.EXPORTS) == names, "the Python binding must mirror the header one to one"


def test_create_validation_and_sizes():
    with pytest.raises(pb.PacError) as e:
        pb.pac_create(0, 768, 128, 96, 3, 32, 16, pb.PAC_BF16)
    assert e.value.status == pb.PAC_ERR_SHAPE
    for bad in [dict(d=770), dict(r=100), dict(C=17), dict(B_max=65)]:
        kw = dict(L=2, d=768, n_max=128, r=96, C=3, B_max=32, N=16)
        kw.update(bad)
        with pytest.raises(pb.PacError) as e:
            pb.pac_create(kw["L"], kw["d"], kw["n_max"], kw["r"], kw["C"], kw["B_max"], kw["N"], pb.PAC_BF16)
        assert e.value.status == pb.PAC_ERR_UNSUPPORTED
    with pytest.raises(pb.PacError) as e:
        pb.pac_create(2, 768, 128, 96, 3, 32, 16, 7)
    assert e.value.status == pb.PAC_ERR_SHAPE
    assert pb.lib().pac_create(None, None) == pb.PAC_ERR_NULL

    ctx = pb.pac_create(12, 768, 128, 96, 3, 32, 4096, pb.PAC_BF16)
    try:
        P = 12 * (2 * 768 * 96 + 96 + 768 + 1) + 768 * 3 + 3
        assert pb.pac_param_count(ctx) == P == 1782159
        assert pb.pac_param_offsets(ctx, 0) == [0, 768 * 96, 768 * 96 + 96, 2 * 768 * 96 + 96, 2 * 768 * 96 + 96 + 768]
        assert pb.pac_param_offsets(ctx, -1)[:2] == [P - 768 * 3 - 3, P - 3]
        with pytest.raises(pb.PacError):
            pb.pac_param_offsets(ctx, 12)
        # storage: tokens x hidden x layers elements per sequence (paper Sec. 5.2), 2 bytes each
        assert pb.pac_cache_bytes(ctx, None, 4096) == 4096 * 128 * 768 * 12 * 2
        assert pb.pac_cache_bytes(ctx, [5, 128, 1], 3) == (5 + 128 + 1) * 768 * 12 * 2
        assert pb.pac_cache_bytes(ctx, [0], 1) == -1 and pb.pac_cache_bytes(ctx, [129], 1) == -1
        assert pb.pac_workspace_bytes(ctx) > 0 and pb.pac_workspace_bytes(ctx) % 256 == 0
    finally:
        pb.pac_destroy(ctx)
    # the paper's storage example: T5-Base, 500 samples of 30 tokens, fp32, below 1 GB
    ctx = pb.pac_create(12, 768, 30, 96, 3, 32, 500, pb.PAC_F32)
    assert pb.pac_cache_bytes(ctx, None, 500) == 552_960_000 < 10 ** 9
    pb.pac_destroy(ctx)
    pb.pac_destroy(None)


def test_formulation_chosen_per_configuration():
    """Host logic: which formulation a configuration runs on (0 per-layer, 1 Gram with single-launch chains,
    2 Gram with layer-by-layer chains)."""
    def path(L, d, n, r, C, B, dtype=pb.PAC_BF16, flags=0):
        ctx = pb.pac_create(L, d, n, r, C, B, 64, dtype, flags)
        try:
            return pb.pac_step_path(ctx)
        finally:
            pb.pac_destroy(ctx)

    assert path(12, 768, 128, 96, 3, 32) == 1            # T5-Base-shaped
    assert path(24, 1024, 128, 128, 2, 32) == 1          # Large-shaped: the chain kernels' LDS just fits
    assert path(32, 4096, 256, 256, 4, 16) == 2          # LLaMA-7B-shaped: r > 128
    assert path(12, 768, 128, 160, 3, 32) == 2
    assert path(40, 1024, 128, 128, 2, 32) == 2          # too many layers for the LDS-resident chains
    assert path(12, 768, 128, 96, 3, 32, pb.PAC_F32) == 0
    assert path(12, 768, 128, 96, 3, 32, flags=pb.PAC_FLAG_PER_LAYER) == 0
    assert path(12, 768, 128, 96, 3, 32, flags=pb.PAC_FLAG_LAYER_CHAIN) == 2
    assert path(32, 4096, 1024, 512, 2, 8) == 2          # long-sequence configuration
    assert path(12, 768, 128, 320, 3, 32) == 2
    assert path(12, 768, 128, 288, 3, 32) == 0           # above 256 only in multiples of 64
    assert path(12, 768, 128, 544, 3, 32) == 0           # wider than the Gram path takes
    assert path(40, 1024, 128, 384, 2, 32) == 0          # above 256 only up to 32 layers
    assert path(80, 4096, 64, 256, 3, 8) == 0            # more layers than the wide path's vector part deals with
    assert pb.lib().pac_step_path(None) == -1


def test_argument_errors_are_caught_before_any_launch():
    """Fake (never dereferenced) device addresses: every call below must fail on the host."""
    ctx = pb.pac_create(2, 64, 16, 32, 3, 4, 8, pb.PAC_BF16)
    lib = pb.lib()
    dev = 0x7000_0000_0000          # aligned, never touched
    ids = np.array([0, 1], dtype=np.int64)
    idp = ids.ctypes.data_as(C.c_void_p)
    big = 1 << 30
    try:
        assert lib.pac_cache_fill(ctx, None, big, idp, 2, dev, pb.PAC_F32, None, None) == pb.PAC_ERR_NULL
        assert lib.pac_cache_fill(ctx, dev + 8, big, idp, 2, dev, pb.PAC_F32, None, None) == pb.PAC_ERR_ALIGN
        assert lib.pac_cache_fill(ctx, dev, big, idp, -1, dev, pb.PAC_F32, None, None) == pb.PAC_ERR_RANGE
        assert lib.pac_cache_fill(ctx, dev, big, idp, 2, dev, 9, None, None) == pb.PAC_ERR_SHAPE
        assert lib.pac_cache_fill(ctx, dev, 100, idp, 2, dev, pb.PAC_F32, None, None) == pb.PAC_ERR_WORKSPACE
        bad_ids = np.array([0, 8], dtype=np.int64)
        assert lib.pac_cache_fill(ctx, dev, big, bad_ids.ctypes.data_as(C.c_void_p), 2, dev, pb.PAC_F32, None,
                                  None) == pb.PAC_ERR_RANGE
        dup = np.array([3, 3], dtype=np.int64)
        assert lib.pac_cache_fill(ctx, dev, big, dup.ctypes.data_as(C.c_void_p), 2, dev, pb.PAC_F32, None,
                                  None) == pb.PAC_ERR_RANGE
        lens = np.array([4, 17], dtype=np.int32)
        assert lib.pac_cache_fill(ctx, dev, big, idp, 2, dev, pb.PAC_F32, lens.ctypes.data_as(C.c_void_p),
                                  None) == pb.PAC_ERR_RANGE
        assert lib.pac_cache_fill(ctx, dev, big, idp, 0, dev, pb.PAC_F32, None, None) == pb.PAC_OK
        with pytest.raises(pb.PacError) as e:
            pb.pac_cache_lookup(ctx, 0)
        assert e.value.status == pb.PAC_ERR_STATE

        ws = pb.pac_workspace_bytes(ctx)
        call = lambda **k: lib.pac_adapter_loss_grad(
            ctx, k.get("cache", dev), k.get("ids", idp), k.get("B", 2), k.get("labels", dev),
            k.get("params", dev), k.get("ws", dev), k.get("ws_bytes", ws), k.get("loss", dev), None, None, None)
        assert call(cache=None) == pb.PAC_ERR_NULL
        assert call(loss=None) == pb.PAC_ERR_NULL
        assert call(ws=dev + 16) == pb.PAC_ERR_ALIGN
        assert call(ws_bytes=ws - 1) == pb.PAC_ERR_WORKSPACE
        assert call(B=0) == pb.PAC_ERR_RANGE and call(B=5) == pb.PAC_ERR_RANGE
        assert call() == pb.PAC_ERR_STATE            # samples 0 and 1 were never filled
        hp = pb.pac_adamw(1e-3, 0.9, 0.999, 1e-8, 0.01)
        st = C.c_int64(0)
        stepcall = lambda hp_, st_: lib.pac_adapter_step(ctx, dev, idp, 2, dev, dev, dev, dev, st_, hp_, dev, ws,
                                                         dev, None, None)
        assert stepcall(None, C.byref(st)) == pb.PAC_ERR_NULL
        assert stepcall(C.byref(pb.pac_adamw(1e-3, 1.0, 0.999, 1e-8, 0.0)), C.byref(st)) == pb.PAC_ERR_RANGE
        assert stepcall(C.byref(hp), C.byref(C.c_int64(-1))) == pb.PAC_ERR_RANGE
        assert stepcall(C.byref(hp), C.byref(st)) == pb.PAC_ERR_STATE and st.value == 0
        # measurement probes: argument errors before any launch
        assert lib.pac_probe_hbm_read(None, 1024, dev, None) == pb.PAC_ERR_NULL
        assert lib.pac_probe_hbm_read(dev, 0, dev, None) == pb.PAC_ERR_RANGE
        assert lib.pac_probe_hbm_read(dev, 1000, dev, None) == pb.PAC_ERR_RANGE
        assert lib.pac_probe_hbm_read(dev + 8, 1024, dev, None) == pb.PAC_ERR_ALIGN
        assert lib.pac_probe_mfma_bf16(0, dev, None) == pb.PAC_ERR_RANGE
        assert lib.pac_probe_mfma_bf16(10, None, None) == pb.PAC_ERR_NULL
        assert pb.pac_probe_mfma_flops(1) == 4 * 2 * 32 * 32 * 16 * 4 * 1024
        assert lib.pac_profile_end(ctx, 32, None, None, None) == pb.PAC_ERR_NULL
        for s in range(9):
            assert isinstance(pb.status_str(s), str) and pb.status_str(s)
    finally:
        pb.pac_destroy(ctx)


def test_ladder_argument_errors_are_caught_before_any_launch():
    """The ladder's calls (include/pac_ladder.h) on fake device addresses: every call must fail on the host."""
    ctx = pb.pac_create(2, 64, 16, 32, 3, 4, 8, pb.PAC_BF16)
    lib = pb.lib()
    dev = 0x7000_0000_0000
    ids = np.array([0, 1], dtype=np.int64)
    idp = ids.ctypes.data_as(C.c_void_p)
    try:
        w, d, f, L, Cc = 32, 64, 128, 2, 3
        per_layer = d * w + w + 2 * w + 3 * w * w + 3 * w + w * w + w + 2 * w + w * f + f + f * w + w + 4
        assert pb.pac_ladder_param_count(ctx) == L * per_layer + w * d + d + d * Cc + Cc
        assert lib.pac_ladder_param_count(None) == -1
        assert pb.pac_ladder_workspace_bytes(ctx, 3) == -1        # 32 / 3 is not a whole head width
        assert pb.pac_ladder_workspace_bytes(ctx, 16) == -1       # head width 2 is not supported
        ws = pb.pac_ladder_workspace_bytes(ctx, 4)
        assert ws > 0 and ws % 256 == 0
        call = lambda **k: lib.pac_ladder_loss_grad(
            ctx, k.get("cache", dev), k.get("ids", idp), k.get("B", 2), k.get("labels", dev), k.get("heads", 4),
            k.get("params", dev), k.get("ws", dev), k.get("ws_bytes", ws), k.get("loss", dev), None, None, None)
        assert call(cache=None) == pb.PAC_ERR_NULL and call(loss=None) == pb.PAC_ERR_NULL
        assert call(params=dev + 4) == pb.PAC_ERR_ALIGN and call(ws=dev + 16) == pb.PAC_ERR_ALIGN
        assert call(heads=3) == pb.PAC_ERR_UNSUPPORTED
        assert call(ws_bytes=ws - 1) == pb.PAC_ERR_WORKSPACE
        assert call(B=0) == pb.PAC_ERR_RANGE and call(B=5) == pb.PAC_ERR_RANGE
        assert call() == pb.PAC_ERR_STATE                         # samples 0 and 1 were never filled
        hp = pb.pac_adamw(1e-3, 0.9, 0.999, 1e-8, 0.01)
        st = C.c_int64(0)
        step = lambda hp_, st_, m_=dev: lib.pac_ladder_step(ctx, dev, idp, 2, dev, 4, dev, m_, dev, st_, hp_, dev, ws, dev,
                                                            None, None)
        assert step(None, C.byref(st)) == pb.PAC_ERR_NULL and step(C.byref(hp), C.byref(st), None) == pb.PAC_ERR_NULL
        assert step(C.byref(pb.pac_adamw(1e-3, 0.9, 1.0, 1e-8, 0.0)), C.byref(st)) == pb.PAC_ERR_RANGE
        assert step(C.byref(hp), C.byref(C.c_int64(-1))) == pb.PAC_ERR_RANGE
        assert step(C.byref(hp), C.byref(st)) == pb.PAC_ERR_STATE and st.value == 0
        assert lib.pac_probe_hbm_update(dev, dev, dev, None, 1024, None) == pb.PAC_ERR_NULL
        assert lib.pac_probe_hbm_update(dev, dev, dev, dev, 1022, None) == pb.PAC_ERR_RANGE
        assert lib.pac_probe_hbm_update(dev, dev + 8, dev, dev, 1024, None) == pb.PAC_ERR_ALIGN
    finally:
        pb.pac_destroy(ctx)
