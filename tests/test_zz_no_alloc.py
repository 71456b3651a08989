"""The entry point that allocates nothing (pac_adapter_step_static: the workspace is a device array inside
the library) against pac_adapter_step on a caller-supplied workspace: same kernels, same order of every
reduction, so parameters, optimizer state, loss and gradients must agree bit for bit.  Two calls in a row on
one context, the second on a smaller batch (the static array still holds the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2408_10746_amd import binding as pb
from paper_2408_10746_amd import inputs
from paper_2408_10746_amd.inputs import Workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("w", [
    Workload("na_f32", L=4, d=256, n_max=64, B=8, r=32, C=2, N=8, cache_dtype="f32"),          # the Tiny shape
    Workload("na_bf16", L=5, d=128, n_max=70, B=4, r=64, C=3, N=4, cache_dtype="bf16", len_lo=20),
    Workload("na_wide", L=3, d=160, n_max=37, B=5, r=160, C=3, N=5, cache_dtype="bf16", len_lo=9),
], ids=lambda w: w.name)
def test_static_workspace_step_matches_workspace_step(w):
    from paper_2408_10746_amd.runtime import Session, _stream_handle
    lens = inputs.lengths(w)
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    labels = torch.from_numpy(inputs.labels(w)[ids]).cuda()
    p0 = inputs.random_params(w, up_scale=0.5)

    def run(static):
        sess = Session(w, lens=lens)
        assert sess.ws_bytes <= pb.PAC_STATIC_WORKSPACE_BYTES
        sess.cache_fill(ids, acts, lens)
        sess.set_params(p0)
        out = []
        for sel in (ids, ids[1:w.B // 2 + 1]):              # second call: fewer samples, other token count
            lab = labels[torch.from_numpy(sel).cuda()].contiguous()
            sess.grads.zero_()
            if static:
                sess.step_count = pb.pac_adapter_step_static(
                    sess.ctx, sess.cache.data_ptr(), sel, lab.data_ptr(), sess.params.data_ptr(), sess.m.data_ptr(),
                    sess.v.data_ptr(), sess.step_count, sess.hp, sess.loss.data_ptr(), sess.grads.data_ptr(),
                    _stream_handle())
            else:
                sess.step(sel, lab)
            torch.cuda.synchronize()
            out.append([t.clone() for t in (sess.loss, sess.grads, sess.params, sess.m, sess.v)])
        assert sess.step_count == 2
        return out

    ref = run(False)
    got = run(True)
    for call, (a, b) in enumerate(zip(ref, got)):
        for name, x, y in zip(("loss", "grads", "params", "m", "v"), a, b):
            assert torch.equal(x, y), (w.name, call, name)
    assert torch.isfinite(got[1][0]).all() and got[1][1].abs().max() > 0


def test_static_workspace_rejects_configurations_beyond_its_size():
    w = inputs.WORKLOADS["t5base"]
    ctx = pb.pac_create(w.L, w.d, w.n_max, w.r, w.C, w.B, 64, pb.PAC_BF16)
    try:
        assert pb.pac_workspace_bytes(ctx) > pb.PAC_STATIC_WORKSPACE_BYTES
        dev = torch.zeros(64, device="cuda")
        with pytest.raises(pb.PacError) as e:
            pb.pac_adapter_step_static(ctx, dev.data_ptr(), [0], dev.data_ptr(), dev.data_ptr(), dev.data_ptr(),
                                       dev.data_ptr(), 0, pb.pac_adamw(1e-3, 0.9, 0.999, 1e-8, 0.01), dev.data_ptr())
        assert e.value.status == pb.PAC_ERR_WORKSPACE
    finally:
        pb.pac_destroy(ctx)
