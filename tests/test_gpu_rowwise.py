"""The two HBM-bound row kernels on their own: the standalone online-softmax merge and D = rowsum(dO o O).
Both walk the (batch, row, head) triples of a tensor with a cursor that is split once and then advanced by
carries, so the shapes here are chosen for the carries: head counts that are not powers of two, a single row,
more head rows than one pass of the grid covers (the cursor then advances several times per lane), strided
views with poisoned padding, bf16 and fp32 partial results, dead (-inf) rows on either side of the merge."""
import numpy as np
import pytest

from oracle import burst_oracle as oc
from paper_2509_19836_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu

SHAPES = [(1, 1, 1, 64), (3, 77, 5, 64), (2, 1000, 3, 128), (1, 4099, 7, 128), (5, 33, 6, 64), (2, 19, 12, 128)]


def _strided(torch, shape, dtype, pad_heads, pad_rows, fill):
    """A [B, S, H, d] view into a larger buffer whose padding holds `fill`."""
    B, S, H, d = shape
    buf = torch.full((B, S + pad_rows, H + pad_heads, d), fill, device="cuda", dtype=dtype)
    return buf, buf[:, :S, :H, :]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("part_dtype", ["f32", "bf16"])
def test_merge_shapes_and_strides(lib, shape, part_dtype):
    import torch
    B, S, H, d = shape
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 61000 + S * 7 + H))
    O_acc = rng.standard_normal(shape).astype(np.float32)
    lse_acc = rng.uniform(-3.0, 5.0, (B, H, S)).astype(np.float32)
    lse_acc[rng.random((B, H, S)) < 0.25] = -np.inf
    part_bits = wl.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))
    O_part = hp.widen(part_bits).astype(np.float32)   # bf16-representable, so both dtypes see the same values
    lse_part = rng.uniform(-3.0, 5.0, (B, H, S)).astype(np.float32)
    lse_part[rng.random((B, H, S)) < 0.25] = -np.inf
    O_ref, lse_ref = oc.mha_lse_merge(O_acc.astype(np.float64), lse_acc.astype(np.float64), O_part.astype(np.float64),
                                      lse_part.astype(np.float64))
    # a dead running row may hold anything; a dead partial row too
    dead_acc = np.transpose(lse_acc == -np.inf, (0, 2, 1))
    O_acc[dead_acc] = np.nan
    acc_buf, o_acc = _strided(torch, shape, torch.float32, 1, 2, 777.0)
    o_acc.copy_(torch.from_numpy(O_acc))
    pdt = torch.float32 if part_dtype == "f32" else torch.bfloat16
    part_buf, o_part = _strided(torch, shape, pdt, 2, 1, 555.0)
    o_part.copy_(torch.from_numpy(O_part).to(pdt))
    out_buf, o_out = _strided(torch, shape, torch.bfloat16, 1, 1, 333.0)
    l_acc = torch.from_numpy(lse_acc).cuda()
    l_part = torch.from_numpy(lse_part).cuda()
    shp = lib.shape(B, H, 1, d, S, S, 1.0)
    lib.burst_attn_lse_merge(shp, o_acc, l_acc, o_part, l_part, o_out_cast=o_out)
    torch.cuda.synchronize()
    got = o_acc.cpu().numpy().astype(np.float64)
    both_dead = dead_acc & np.transpose(lse_part == -np.inf, (0, 2, 1))
    live = ~both_dead
    assert np.isfinite(got[live]).all()
    assert np.abs(got[live] - O_ref[live]).max() <= 1e-4 * max(1.0, np.abs(O_ref[live]).max())
    assert hp.lse_err(l_acc.cpu().numpy(), lse_ref) <= 1e-4
    assert torch.equal(o_out[torch.from_numpy(live)], o_acc[torch.from_numpy(live)].to(torch.bfloat16))
    # padding untouched
    assert (acc_buf[:, S:] == 777.0).all() and (acc_buf[:, :, H:] == 777.0).all()
    assert (out_buf[:, S:] == 333.0).all() and (out_buf[:, :, H:] == 333.0).all()


@pytest.mark.parametrize("shape", SHAPES)
def test_preprocess_shapes_and_strides(lib, shape):
    import torch
    B, S, H, d = shape
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 62000 + S * 7 + H))
    O = rng.standard_normal(shape).astype(np.float32)
    g_bits = wl.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))
    _, o = _strided(torch, shape, torch.float32, 3, 1, float("nan"))
    o.copy_(torch.from_numpy(O))
    _, g = _strided(torch, shape, torch.bfloat16, 1, 4, float("nan"))
    g.copy_(hp.dev_bf16(g_bits))
    dvec = torch.full((B, H + 1, S + 8), 99.0, device="cuda", dtype=torch.float32)
    shp = lib.shape(B, H, 1, d, S, S, 1.0)
    lib.burst_attn_preprocess_bwd(shp, o, g, dvec[:, :H, :S])
    torch.cuda.synchronize()
    D_ref = oc.mha_preprocess_bwd(hp.widen(g_bits), O.astype(np.float64))
    got = dvec[:, :H, :S].cpu().numpy()
    assert np.abs(got - D_ref).max() <= 1e-4 * max(1.0, np.abs(D_ref).max())
    assert (dvec[:, H:] == 99.0).all() and (dvec[:, :, S:] == 99.0).all()


def test_more_head_rows_than_one_pass_of_the_grid(lib):
    """1.28 million head rows of 128: more than the grid's 65536 blocks x 16 head rows cover in one pass, so lanes
    advance their cursors; D and the merge on sampled rows against the oracle, all of D against a float32
    restatement."""
    import torch
    B, S, H, d = 2, 40000, 16, 128
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.BASE_SEED + 63000)
    o = torch.randn(B, S, H, d, device="cuda", generator=gen)
    g = torch.randn(B, S, H, d, device="cuda", generator=gen).to(torch.bfloat16)
    dvec = torch.empty(B, H, S, device="cuda")
    shp = lib.shape(B, H, 1, d, S, S, 1.0)
    lib.burst_attn_preprocess_bwd(shp, o, g, dvec)
    torch.cuda.synchronize()
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 63001))
    rows = np.unique(np.concatenate([[0, 1, S - 2, S - 1], rng.integers(0, S, 400)]))
    o_h, g_h = o[:, rows].cpu().numpy().astype(np.float64), g[:, rows].float().cpu().numpy().astype(np.float64)
    D_ref = oc.mha_preprocess_bwd(g_h, o_h)
    assert np.abs(dvec[:, :, rows].cpu().numpy() - D_ref).max() <= 1e-4 * np.abs(D_ref).max()
    # every row at once against a float32 restatement on the GPU (not the oracle: a size check of the cursor)
    whole = (o * g.float()).sum(-1).permute(0, 2, 1)
    assert (dvec - whole).abs().max().item() <= 1e-3

    o_acc = torch.randn(B, S, H, d, device="cuda", generator=gen)
    o_part = torch.randn(B, S, H, d, device="cuda", generator=gen)
    l_acc = torch.randn(B, H, S, device="cuda", generator=gen)
    l_part = torch.randn(B, H, S, device="cuda", generator=gen)
    acc0, lacc0 = o_acc[:, rows].cpu().numpy().astype(np.float64), l_acc[:, :, rows].cpu().numpy().astype(np.float64)
    lib.burst_attn_lse_merge(shp, o_acc, l_acc, o_part, l_part)
    torch.cuda.synchronize()
    O_ref, lse_ref = oc.mha_lse_merge(acc0, lacc0, o_part[:, rows].cpu().numpy().astype(np.float64),
                                      l_part[:, :, rows].cpu().numpy().astype(np.float64))
    assert np.abs(o_acc[:, rows].cpu().numpy() - O_ref).max() <= 1e-4 * np.abs(O_ref).max()
    assert np.abs(l_acc[:, :, rows].cpu().numpy() - lse_ref).max() <= 1e-4
