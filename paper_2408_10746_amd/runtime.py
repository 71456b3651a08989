"""Device-memory plumbing around the C ABI for tests, the smoke check and the benchmark.

PyTorch is used for nothing but allocating device buffers, host<->device copies
and the stream handle; every computation of the path happens inside libpac.so.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as pb
from .inputs import Workload


def _stream_handle() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


class Session:
    """Owns the device buffers of one configuration (cache, workspace, params, optimizer state)."""

    def __init__(self, w: Workload, cache_samples: int | None = None, lens=None, device: str = "cuda:0",
                 flags: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("libpac needs a GPU: no HIP device is visible")
        self.w = w
        self.dev = torch.device(device)
        self.dtype = pb.PAC_BF16 if w.cache_dtype == "bf16" else pb.PAC_F32
        self.ctx = pb.pac_create(w.L, w.d, w.n_max, w.r, w.C, w.B, w.N, self.dtype, flags)
        self.P = pb.pac_param_count(self.ctx)
        n = w.N if cache_samples is None else cache_samples
        self.cache_bytes = pb.pac_cache_bytes(self.ctx, lens, n)
        assert self.cache_bytes > 0
        self.cache = torch.empty(self.cache_bytes, dtype=torch.uint8, device=self.dev)
        self.ws_bytes = pb.pac_workspace_bytes(self.ctx)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        self.params = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.m = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.v = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.grads = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.dev)
        self.logits = torch.zeros(w.B * w.C, dtype=torch.float32, device=self.dev)
        self.step_count = 0
        self.hp = pb.pac_adamw(1e-3, 0.9, 0.999, 1e-8, 0.01)

    def close(self):
        if self.ctx:
            pb.pac_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- state -----------------------------------------------------------
    def set_params(self, p: np.ndarray) -> None:
        self.params.copy_(torch.from_numpy(np.ascontiguousarray(p, dtype=np.float32)))
        self.m.zero_()
        self.v.zero_()
        self.step_count = 0

    # ---- the two calls ---------------------------------------------------
    def cache_fill(self, sample_ids, acts, lens=None) -> None:
        """acts: device tensor [count][L][n_max][d], float32 or bfloat16 (or a numpy float32 array)."""
        if isinstance(acts, np.ndarray):
            acts = torch.from_numpy(np.ascontiguousarray(acts, dtype=np.float32)).to(self.dev)
        assert acts.is_contiguous() and acts.device.type == "cuda"
        dt = pb.PAC_BF16 if acts.dtype == torch.bfloat16 else pb.PAC_F32
        assert acts.dtype in (torch.bfloat16, torch.float32)
        pb.pac_cache_fill(self.ctx, self.cache.data_ptr(), self.cache_bytes, sample_ids, acts.data_ptr(), dt,
                          lens, _stream_handle())

    def loss_grad(self, sample_ids, labels_dev, want_grads: bool = True, want_logits: bool = True) -> None:
        pb.pac_adapter_loss_grad(self.ctx, self.cache.data_ptr(), sample_ids, labels_dev.data_ptr(),
                                 self.params.data_ptr(), self.ws.data_ptr(), self.ws_bytes,
                                 self.loss.data_ptr(), self.logits.data_ptr() if want_logits else None,
                                 self.grads.data_ptr() if want_grads else None, _stream_handle())

    def step(self, sample_ids, labels_dev, keep_grads: bool = True) -> None:
        self.step_count = pb.pac_adapter_step(
            self.ctx, self.cache.data_ptr(), sample_ids, labels_dev.data_ptr(), self.params.data_ptr(),
            self.m.data_ptr(), self.v.data_ptr(), self.step_count, self.hp, self.ws.data_ptr(), self.ws_bytes,
            self.loss.data_ptr(), self.grads.data_ptr() if keep_grads else None, _stream_handle())

    # ---- read-back -------------------------------------------------------
    def cache_block(self, sample_id: int) -> np.ndarray:
        """Stored values of one sample: uint16 bf16 bits or float32, [L][len][d]."""
        off, ln = pb.pac_cache_lookup(self.ctx, sample_id)
        es = 2 if self.dtype == pb.PAC_BF16 else 4
        n = self.w.L * ln * self.w.d
        raw = self.cache[off * es:(off + n) * es].cpu().numpy()
        return raw.view(np.uint16 if es == 2 else np.float32).reshape(self.w.L, ln, self.w.d)


class LadderSession(Session):
    """The same cache trained through the paper's default architecture (include/pac_ladder.h): own parameter vector
    and workspace, the ladder's two calls."""

    def __init__(self, w: Workload, heads: int, cache_samples: int | None = None, lens=None, device: str = "cuda:0"):
        super().__init__(w, cache_samples=cache_samples, lens=lens, device=device)
        self.heads = heads
        self.P = pb.pac_ladder_param_count(self.ctx)
        self.ws_bytes = pb.pac_ladder_workspace_bytes(self.ctx, heads)
        if self.P <= 0 or self.ws_bytes <= 0:
            raise ValueError("configuration not supported by the ladder path")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        self.params = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.m = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.v = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.grads = torch.zeros(self.P, dtype=torch.float32, device=self.dev)

    def loss_grad(self, sample_ids, labels_dev, want_grads: bool = True, want_logits: bool = True) -> None:
        pb.pac_ladder_loss_grad(self.ctx, self.cache.data_ptr(), sample_ids, labels_dev.data_ptr(), self.heads,
                                self.params.data_ptr(), self.ws.data_ptr(), self.ws_bytes, self.loss.data_ptr(),
                                self.logits.data_ptr() if want_logits else None,
                                self.grads.data_ptr() if want_grads else None, _stream_handle())

    def step(self, sample_ids, labels_dev, keep_grads: bool = True) -> None:
        self.step_count = pb.pac_ladder_step(
            self.ctx, self.cache.data_ptr(), sample_ids, labels_dev.data_ptr(), self.heads, self.params.data_ptr(),
            self.m.data_ptr(), self.v.data_ptr(), self.step_count, self.hp, self.ws.data_ptr(), self.ws_bytes,
            self.loss.data_ptr(), self.grads.data_ptr() if keep_grads else None, _stream_handle())


class TieredSession(Session):
    """The same buffers with the cache in pinned host memory and two device windows: batch k + 1 is reloaded on a
    copy stream while batch k trains on the compute stream (events order the two; default stream priorities)."""

    def __init__(self, w: Workload, cache_samples: int | None = None, lens=None, device: str = "cuda:0", flags: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("libpac needs a GPU: no HIP device is visible")
        self.w = w
        self.dev = torch.device(device)
        self.dtype = pb.PAC_BF16 if w.cache_dtype == "bf16" else pb.PAC_F32
        self.ctx = pb.pac_create(w.L, w.d, w.n_max, w.r, w.C, w.B, w.N, self.dtype, flags)
        self.P = pb.pac_param_count(self.ctx)
        n = w.N if cache_samples is None else cache_samples
        self.cache_bytes = pb.pac_cache_bytes(self.ctx, lens, n)
        assert self.cache_bytes > 0
        self.host_cache = torch.empty(self.cache_bytes, dtype=torch.uint8, pin_memory=True)
        self.window_bytes = pb.pac_tier_window_bytes(self.ctx)
        self.windows = [torch.empty(self.window_bytes, dtype=torch.uint8, device=self.dev) for _ in range(2)]
        self.copy_stream = torch.cuda.Stream(device=self.dev)
        self.ready = [torch.cuda.Event() for _ in range(2)]
        self.free = [torch.cuda.Event() for _ in range(2)]
        for e in self.free:
            e.record()
        self.ws_bytes = pb.pac_workspace_bytes(self.ctx)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        self.params = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.m = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.v = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.grads = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.dev)
        self.logits = torch.zeros(w.B * w.C, dtype=torch.float32, device=self.dev)
        self.step_count = 0
        self.hp = pb.pac_adamw(1e-3, 0.9, 0.999, 1e-8, 0.01)

    def cache_fill(self, sample_ids, acts, lens=None) -> None:
        if isinstance(acts, np.ndarray):
            acts = torch.from_numpy(np.ascontiguousarray(acts, dtype=np.float32)).to(self.dev)
        assert acts.is_contiguous() and acts.device.type == "cuda"
        dt = pb.PAC_BF16 if acts.dtype == torch.bfloat16 else pb.PAC_F32
        pb.pac_tier_fill(self.ctx, self.host_cache.data_ptr(), self.cache_bytes, sample_ids, acts.data_ptr(), dt, lens,
                         self.windows[0].data_ptr(), self.window_bytes, _stream_handle())
        self.free[0].record()

    def prefetch(self, k: int, sample_ids) -> None:
        """Reload the batch into window k % 2 on the copy stream, once the step that last read that window is done."""
        slot = k % 2
        self.copy_stream.wait_event(self.free[slot])
        pb.pac_tier_stage(self.ctx, self.host_cache.data_ptr(), sample_ids, self.windows[slot].data_ptr(), self.window_bytes,
                          int(self.copy_stream.cuda_stream))
        self.ready[slot].record(self.copy_stream)

    def step_staged(self, k: int, sample_ids, labels_dev, keep_grads: bool = True) -> None:
        slot = k % 2
        torch.cuda.current_stream().wait_event(self.ready[slot])
        self.step_count = pb.pac_adapter_step_staged(
            self.ctx, self.windows[slot].data_ptr(), sample_ids, labels_dev.data_ptr(), self.params.data_ptr(),
            self.m.data_ptr(), self.v.data_ptr(), self.step_count, self.hp, self.ws.data_ptr(), self.ws_bytes,
            self.loss.data_ptr(), self.grads.data_ptr() if keep_grads else None, _stream_handle())
        self.free[slot].record()

    def loss_grad_staged(self, k: int, sample_ids, labels_dev) -> None:
        slot = k % 2
        torch.cuda.current_stream().wait_event(self.ready[slot])
        pb.pac_adapter_loss_grad_staged(self.ctx, self.windows[slot].data_ptr(), sample_ids, labels_dev.data_ptr(),
                                        self.params.data_ptr(), self.ws.data_ptr(), self.ws_bytes, self.loss.data_ptr(),
                                        self.logits.data_ptr(), self.grads.data_ptr(), _stream_handle())
        self.free[slot].record()

    def cache_block(self, sample_id: int) -> np.ndarray:
        torch.cuda.synchronize()
        off, ln = pb.pac_cache_lookup(self.ctx, sample_id)
        es = 2 if self.dtype == pb.PAC_BF16 else 4
        n = self.w.L * ln * self.w.d
        raw = self.host_cache[off * es:(off + n) * es].numpy()
        return raw.view(np.uint16 if es == 2 else np.float32).reshape(self.w.L, ln, self.w.d).copy()
