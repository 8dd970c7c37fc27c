"""burst_lm_head_loss_noalloc (the entry point for callers that cannot allocate: it runs on the
library's built-in scratch array) against burst_lm_head_loss with a caller's workspace, through the
C ABI: two calls in a row on the same GPU, the second with a smaller input, each compared with the
workspace entry point on the same inputs (bit for bit: both run the same kernels on the same
values) and with the fp64 oracle to the stated bar."""
import numpy as np
import pytest

from oracle import lm_head_oracle as lm
from paper_2509_19836_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _both(lib, seed, N, d, v, B_s, grad_scale):
    import torch
    Hb, Wb, Y = wl.lm_head_tensors(seed, N, d, v, ignored=1)
    h, w, y = hp.dev_bf16(Hb), hp.dev_bf16(Wb), torch.from_numpy(Y).cuda()
    shp = lib.lm_head_shape(N, d, v, B_s, grad_scale)
    f32 = dict(dtype=torch.float32, device="cuda")
    out = {}
    for name in ("workspace", "noalloc"):
        loss, lse = torch.full((N,), 7.0, **f32), torch.full((N,), 7.0, **f32)
        dh, dw = torch.full((N, d), 5.0, **f32), torch.full((v, d), float("nan"), **f32)
        print(f"lm head {name}: N={N} d={d} v={v} B_s={B_s}", flush=True)
        if name == "workspace":
            ws = torch.empty(lib.burst_lm_head_workspace_bytes(shp), dtype=torch.uint8, device="cuda")
            ws.fill_(0xFF)
            lib.burst_lm_head_loss(shp, h, w, y, loss, ws, lse=lse, d_h=dh, d_w=dw)
        else:
            lib.burst_lm_head_loss_noalloc(shp, h, w, y, loss, lse=lse, d_h=dh, d_w=dw)
        torch.cuda.synchronize()
        out[name] = [t.cpu().numpy() for t in (loss, lse, dh, dw)]
    for a, b in zip(out["workspace"], out["noalloc"]):
        assert np.array_equal(a, b)
    loss_ref, lse_ref, dH_ref, dW_ref = lm.lm_head_loss(hp.widen(Hb), hp.widen(Wb), Y, grad_scale)
    loss, lse, dh, dw = out["noalloc"]
    assert np.abs(loss - loss_ref).max() <= hp.LSE_TOL and np.abs(lse - lse_ref).max() <= hp.LSE_TOL
    assert np.abs(dh - dH_ref).max() <= hp.REL_TOL * np.abs(dH_ref).max()
    assert np.abs(dw - dW_ref).max() <= hp.REL_TOL * np.abs(dW_ref).max()


def test_two_calls_in_a_row_second_one_smaller(lib):
    assert lib.burst_lm_head_static_scratch_bytes() == 64 << 20
    _both(lib, wl.BASE_SEED + 21001, N=700, d=512, v=3000, B_s=512, grad_scale=1.0 / 700)   # two tiles, the last ragged
    _both(lib, wl.BASE_SEED + 21002, N=130, d=256, v=900, B_s=256, grad_scale=1.0)          # smaller in every extent


def test_shape_beyond_the_built_in_scratch_is_refused(lib):
    import torch
    shp = lib.lm_head_shape(256, 256, 128256, 256, 1.0)          # 256 tokens x 128256 words x 6 B > 64 MiB
    assert lib.burst_lm_head_workspace_bytes(shp) > lib.burst_lm_head_static_scratch_bytes()
    h = torch.zeros(256, 256, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(128256, 256, dtype=torch.bfloat16, device="cuda")
    y = torch.zeros(256, dtype=torch.int64, device="cuda")
    loss = torch.full((256,), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(lib.BurstError) as err:
        lib.burst_lm_head_loss_noalloc(shp, h, w, y, loss)
    assert err.value.status == lib.BURST_ERR_SCRATCH
    torch.cuda.synchronize()
    assert (loss == 7.0).all()                                   # nothing was enqueued
