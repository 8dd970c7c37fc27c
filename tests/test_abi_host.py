"""CPU-only checks of the C-ABI boundary: the library loads and exports what the header declares,
the host helpers agree with the oracle's partitions, and invalid arguments are rejected before
anything could reach a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import burst_oracle as oc
from tests import helpers as hp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol(lib):
    header = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include")))
                     if f.endswith(".h"))
    declared = set(re.findall(r"\b(burst_(?:attn|lm_head)_\w+)\s*\(", header))
    assert {"burst_attn_step_fwd", "burst_attn_lse_merge", "burst_attn_step_bwd",
            "burst_attn_preprocess_bwd", "burst_lm_head_loss"} <= declared
    raw = lib.raw()
    for name in sorted(declared):
        assert hasattr(raw, name), f"{name} declared in the header but not exported"
    assert declared == set(lib.EXPORTS)
    assert "gfx950" in lib.burst_attn_version()


def test_struct_layouts_match_the_header(lib):
    # natural C layout of the structs in include/burst_attn.h
    assert C.sizeof(lib.burst_shape_t) == 40
    assert C.sizeof(lib.burst_tensor_t) == 40
    assert C.sizeof(lib.burst_rowvec_t) == 24
    assert C.sizeof(lib.burst_mask_t) == 16 + 32 + 32 + 32
    assert C.sizeof(lib.burst_lm_head_shape_t) == 40


@pytest.mark.parametrize("G,N", [(1, 8), (2, 24), (4, 64), (8, 128)])
def test_mask_helpers_agree_with_oracle_partitions(lib, G, N):
    for kind in ("causal", "zigzag", "striped"):
        for i in range(G):
            for j in range(G):
                m = hp.fill_mask(lib, kind, i, j, G, N)
                qpos, kpos = hp.mask_positions(m, "q"), hp.mask_positions(m, "k")
                assert (qpos == hp.oracle_positions(oc, kind, i, G, N)).all()
                assert (kpos == hp.oracle_positions(oc, kind, j, G, N)).all()
                assert lib.burst_attn_visible_pairs(m) == oc.visible_pairs(qpos, kpos, True)
    m = hp.fill_mask(lib, "full", 0, G - 1, G, N)
    assert lib.burst_attn_visible_pairs(m) == (N // G) ** 2
    for kind in ("causal", "zigzag", "striped"):   # sliding windows
        for window in (1, 3, N // G, N):
            for i, j in ((G - 1, 0), (0, G - 1), (G // 2, G // 2)):
                m = hp.fill_mask(lib, kind, i, j, G, N, window)
                assert lib.burst_attn_visible_pairs(m) == oc.visible_pairs(hp.mask_positions(m, "q"),
                                                                            hp.mask_positions(m, "k"), True, window)
    bad = hp.fill_mask(lib, "full", 0, 0, G, N, 5)   # a window needs a causal mask
    assert lib.burst_attn_visible_pairs(bad) == -1


def test_zigzag_pair_counts_closed_form(lib):
    # every step carries the same work: 2 P^2 pairs, plus P on the device's own shard (Sec. 3.4)
    G, N = 8, 8 * 2 * 96
    P = N // (2 * G)
    for i in range(G):
        for j in range(G):
            got = lib.burst_attn_visible_pairs(lib.burst_attn_fill_zigzag_mask(i, j, G, N))
            assert got == 2 * P * P + (P if i == j else 0)


def test_mask_helper_argument_errors(lib):
    raw = lib.raw()
    m = lib.burst_mask_t()
    assert raw.burst_attn_fill_zigzag_mask(0, 0, 4, 100, 1, C.byref(m)) == lib.BURST_ERR_INVALID_ARG  # 100 % 8
    assert raw.burst_attn_fill_zigzag_mask(4, 0, 4, 64, 1, C.byref(m)) == lib.BURST_ERR_INVALID_ARG
    assert raw.burst_attn_fill_contiguous_mask(0, -1, 4, 64, 1, C.byref(m)) == lib.BURST_ERR_INVALID_ARG
    assert raw.burst_attn_fill_striped_mask(0, 0, 0, 64, 1, C.byref(m)) == lib.BURST_ERR_INVALID_ARG
    assert raw.burst_attn_fill_zigzag_mask(0, 0, 4, 64, 1, None) == lib.BURST_ERR_INVALID_ARG
    bad = lib.burst_mask_t(7, 1, 1, 0, (0, 0), (0, 0), 4, 4, 1)
    assert lib.burst_attn_visible_pairs(bad) == -1
    assert lib.burst_attn_status_string(lib.BURST_ERR_UNSUPPORTED).startswith("unsupported")


def _fake_tensor(lib, dtype=0, ptr=0x10000, strides=(1 << 20, 256, 128)):
    return lib.burst_tensor_t(ptr, dtype, 0, *strides)


def _fake_rowvec(lib, ptr=0x20000):
    return lib.burst_rowvec_t(ptr, 4096, 1024)


def test_invalid_arguments_are_rejected_on_the_host(lib):
    """None of these calls may get as far as a HIP call: they all fail validation first.  The
    pointers are made-up numbers that are never dereferenced."""
    raw = lib.raw()
    ok_shape = lib.shape(1, 2, 2, 128, 64, 64, 0.1)
    t, tf32, rv = _fake_tensor(lib), _fake_tensor(lib, dtype=1), _fake_rowvec(lib)
    r = C.byref

    def fwd(shape=ok_shape, mask=None, q=t, k=t, v=t, o_part=tf32, lse_part=rv, o_acc=None, lse_acc=None):
        ref = lambda x: None if x is None else r(x)
        return raw.burst_attn_step_fwd(ref(shape), ref(mask), ref(q), ref(k), ref(v), ref(o_part), ref(lse_part),
                                       ref(o_acc), ref(lse_acc), None)

    INV, UNS = lib.BURST_ERR_INVALID_ARG, lib.BURST_ERR_UNSUPPORTED
    assert fwd(shape=None) == INV
    assert fwd(q=None) == INV
    assert fwd(o_part=None, lse_part=None) == INV                        # no output requested
    assert fwd(lse_part=None) == INV                                     # o_part without lse_part
    assert fwd(q=_fake_tensor(lib, ptr=0)) == INV                        # null data pointer
    assert fwd(q=_fake_tensor(lib, ptr=0x10008)) == INV                  # misaligned
    assert fwd(k=_fake_tensor(lib, strides=(1 << 20, 252, 128))) == INV  # stride not a multiple of 8
    assert fwd(q=tf32) == UNS                                            # fp32 q not supported
    assert fwd(o_acc=t, lse_acc=rv) == UNS                               # running state must be fp32
    assert fwd(shape=lib.shape(1, 2, 2, 96, 64, 64, 0.1)) == UNS         # head_dim
    assert fwd(shape=lib.shape(1, 3, 2, 128, 64, 64, 0.1)) == INV        # heads not divisible
    assert fwd(shape=lib.shape(1, 2, 2, 128, 64, 64, 0.0)) == INV        # scale
    assert fwd(shape=lib.shape(1, 2, 2, 128, 64, 64, float("nan"))) == INV
    assert fwd(shape=lib.shape(0, 2, 2, 128, 64, 64, 0.1)) == INV
    assert fwd(shape=lib.shape(1, 2, 2, 128, -1, 64, 0.1)) == INV
    assert fwd(mask=lib.burst_mask_t(1, 1, 1, 0, (0, 0), (0, 0), 63, 64, 1)) == INV      # seg_len * nseg != sq
    assert fwd(mask=lib.burst_mask_t(1, 3, 1, 0, (0, 0), (0, 0), 64, 64, 1)) == INV      # nseg
    assert fwd(mask=lib.burst_mask_t(2, 1, 1, 0, (0, 0), (0, 0), 64, 64, 1)) == INV      # mode
    assert fwd(mask=lib.burst_mask_t(1, 1, 1, 0, (0, 0), (0, 0), 64, 64, 0)) == INV      # stride
    assert fwd(mask=lib.burst_mask_t(1, 1, 1, 0, (-5, 0), (0, 0), 64, 64, 1)) == INV     # negative position
    assert fwd(mask=lib.burst_mask_t(1, 1, 1, 0, (1 << 31, 0), (0, 0), 64, 64, 1)) == UNS  # position range
    assert fwd(mask=lib.burst_mask_t(1, 1, 1, 0, (0, 0), (0, 0), 64, 64, 1, -3)) == INV    # negative window
    assert fwd(mask=lib.burst_mask_t(0, 1, 1, 0, (0, 0), (0, 0), 64, 64, 1, 16)) == INV    # window without causal
    assert fwd(k=_fake_tensor(lib, strides=(1 << 40, (1 << 24) + 8, 128))) == UNS          # row stride beyond 2^24

    def blk(q_rows, k_rows, pitch, sq=64, sk=64):
        m = lib.burst_mask_t(1, 1, 1, 0, (0, 0), (0, 0), sq, sk, 1, 0, 0x10000, q_rows, k_rows, pitch)
        return fwd(shape=lib.shape(1, 2, 2, 128, sq, sk, 0.1), mask=m)
    assert blk(128, 128, 1) == INV          # query blocks must be multiples of 256 rows
    assert blk(256, 64, 1) == INV           # key blocks of 128
    assert blk(0, 128, 1) == INV
    assert blk(256, 128, 0) == INV          # pitch below the number of key blocks
    assert blk(256, 128, 3, sk=512) == INV
    assert blk(256, 128, 4096, sq=64 * 4096 + 64) == UNS   # more tiles than the kernels' flag cache holds

    def bwd(dq=tf32, dk=tf32, dv=tf32, flags=0, lse=rv, d=rv, d_o=t):
        ref = lambda x: None if x is None else r(x)
        return raw.burst_attn_step_bwd(r(ok_shape), None, r(t), r(t), r(t), ref(d_o), ref(lse), ref(d), ref(dq), ref(dk),
                                       ref(dv), flags, None)

    assert bwd(dq=None, dk=None, dv=None) == INV
    assert bwd(dv=None) == INV                       # dk without dv
    assert bwd(flags=8) == INV
    assert bwd(lse=None) == INV
    assert bwd(dq=t) == UNS                          # gradients are fp32
    assert bwd(d_o=tf32) == UNS
    assert raw.burst_attn_lse_merge(r(ok_shape), r(tf32), r(rv), r(tf32), None, None, None) == INV
    assert raw.burst_attn_lse_merge(r(ok_shape), r(t), r(rv), r(tf32), r(rv), None, None) == UNS
    assert raw.burst_attn_preprocess_bwd(r(ok_shape), r(tf32), r(tf32), r(rv), None) == UNS
    assert raw.burst_attn_preprocess_bwd(r(ok_shape), r(tf32), r(t), None, None) == INV


def test_outputs_that_overlap_and_unbounded_position_strides_are_rejected(lib):
    """An output descriptor that maps two elements to one address would make work-groups race without
    a trace: refused on the host (inputs may overlap: a zero stride broadcasts).  A position stride is
    bounded before it is multiplied with a segment length."""
    raw = lib.raw()
    shp = lib.shape(2, 4, 4, 128, 64, 64, 0.1)
    r = C.byref
    INV, UNS = lib.BURST_ERR_INVALID_ARG, lib.BURST_ERR_UNSUPPORTED
    tin = _fake_tensor(lib, strides=(0, 512, 0))                       # input broadcast over batch and heads: fine
    good = _fake_tensor(lib, dtype=1, strides=(64 * 512, 512, 128))     # [B, S, H, D] packed
    heads_first = _fake_tensor(lib, dtype=1, strides=(4 * 64 * 128, 128, 64 * 128))   # [B, H, S, D] described by strides
    rv = lib.burst_rowvec_t(0x20000, 4 * 64, 64)

    def fwd(o_part=good, lse_part=rv, mask=None):
        return raw.burst_attn_step_fwd(r(shp), None if mask is None else r(mask), r(tin), r(tin), r(tin), r(o_part), r(lse_part),
                                       None, None, None)
    # (the good descriptors get as far as the launch, which needs a GPU: only refusals are asserted here)
    for bad in (_fake_tensor(lib, dtype=1, strides=(64 * 512, 512, 64)),        # heads 64 apart, 128 wide
                _fake_tensor(lib, dtype=1, strides=(64 * 512, 256, 128)),       # rows closer than 4 heads of 128
                _fake_tensor(lib, dtype=1, strides=(64 * 512, 0, 128)),         # every row on the same address
                _fake_tensor(lib, dtype=1, strides=(0, 512, 128)),              # both batch entries on the same address
                _fake_tensor(lib, dtype=1, strides=(4 * 64 * 128, 128, 63 * 128 + 64))):   # [B,H,S,D] with heads too close
        assert fwd(o_part=bad) == INV
    assert fwd(lse_part=lib.burst_rowvec_t(0x20000, 4 * 64, 32)) == INV         # heads of 64 rows, 32 apart
    assert fwd(lse_part=lib.burst_rowvec_t(0x20000, 64, 64)) == INV             # batch entries on top of the heads

    def bwd(dq=good, dk=good, dv=good):
        return raw.burst_attn_step_bwd(r(shp), None, r(tin), r(tin), r(tin), r(tin), r(rv), r(rv), r(dq), r(dk), r(dv), 0, None)
    overl = _fake_tensor(lib, dtype=1, strides=(64 * 512, 512, 64))
    assert bwd(dq=overl) == INV and bwd(dk=overl) == INV and bwd(dv=overl) == INV
    assert raw.burst_attn_lse_merge(r(shp), r(overl), r(rv), r(good), r(rv), None, None) == INV
    assert raw.burst_attn_lse_merge(r(shp), r(good), r(rv), r(good), r(rv), r(_fake_tensor(lib, strides=(64 * 512, 512, 64))), None) == INV
    assert raw.burst_attn_preprocess_bwd(r(shp), r(good), r(tin), r(lib.burst_rowvec_t(0x20000, 4 * 64, 32)), None) == INV
    # a position stride so large that stride * seg_len would wrap int64
    m = lib.burst_mask_t(1, 1, 1, 0, (0, 0), (0, 0), 64, 64, (1 << 62) + 1)
    assert fwd(mask=m) == UNS
    assert lib.raw().burst_attn_tile_class(r(m), 0, 64, 0, 64, 0) == UNS
    assert heads_first.stride_h == 64 * 128   # (descriptor kept for the GPU test of the same layout)


def test_empty_query_chunk_returns_ok_without_a_launch(lib):
    raw = lib.raw()
    t, tf32, rv = _fake_tensor(lib), _fake_tensor(lib, dtype=1), _fake_rowvec(lib)
    shp = lib.shape(1, 2, 2, 128, 0, 64, 0.1)
    assert raw.burst_attn_step_fwd(C.byref(shp), None, C.byref(t), C.byref(t), C.byref(t), C.byref(tf32), C.byref(rv),
                                   None, None, None) == lib.BURST_OK
    assert raw.burst_attn_lse_merge(C.byref(shp), C.byref(tf32), C.byref(rv), C.byref(tf32), C.byref(rv), None,
                                    None) == lib.BURST_OK
    assert raw.burst_attn_preprocess_bwd(C.byref(shp), C.byref(tf32), C.byref(t), C.byref(rv), None) == lib.BURST_OK


def test_binding_refuses_to_load_without_the_library(tmp_path, monkeypatch):
    """There is no CPU fallback: importing the binding without a built library raises."""
    import importlib.util
    src = os.path.join(ROOT, "paper_2509_19836_amd", "binding.py")
    dst = tmp_path / "binding_copy.py"
    dst.write_text(open(src).read())
    spec = importlib.util.spec_from_file_location("binding_copy", dst)
    mod = importlib.util.module_from_spec(spec)
    with pytest.raises(ImportError, match="no CPU or PyTorch fallback"):
        spec.loader.exec_module(mod)


def test_workload_generators_are_seeded_and_exact():
    from paper_2509_19836_amd import workloads as wl
    w = wl.WORKLOADS[1]
    a, b = wl.host_tensors(w, 1), wl.host_tensors(w, 1)
    for n in a:
        assert (a[n][1] == b[n][1]).all()
    x = np.array([1.0, 1.00390625, -2.5, 3.1415927, 1e-30], dtype=np.float32)
    bits = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[2] == -2.5
    assert back[1] == 1.0            # 1 + 2^-8 is a tie: rounds to even
    assert abs(back[3] - 3.140625) < 1e-6
    assert (wl.bf16_bits_to_f64(bits) == back.astype(np.float64)).all()
    w4 = wl.Workload("t", 2, 4, 4, 128, 64, 2, "full", True)
    t4 = wl.host_tensors(w4, 4)
    stds = t4["q"][0].std(axis=(1, 3))
    assert stds.min() > 0.4 and stds.max() < 2.2 and stds.std() > 0.05


def _custom_mask(lib, q_pos, k_pos, q_len, k_len, stride, causal=True, q_nseg=None, k_nseg=None):
    """q_pos / k_pos: start of the first piece, or of the first two (their distance is the period of
    q_nseg / k_nseg pieces)."""
    m = lib.burst_mask_t()
    m.mode = lib.BURST_MASK_CAUSAL if causal else lib.BURST_MASK_FULL
    m.q_nseg, m.k_nseg = q_nseg or len(q_pos), k_nseg or len(k_pos)
    for s, p in enumerate(q_pos):
        m.q_seg_pos[s] = p
    for s, p in enumerate(k_pos):
        m.k_seg_pos[s] = p
    m.q_seg_len, m.k_seg_len, m.pos_stride = q_len, k_len, stride
    return m


def _tile_logic_masks(lib):
    """Masks with segment lengths that are and are not multiples of the tile sizes, one and two
    segments per axis, unit and larger position strides, segments in either position order."""
    out = []
    for G, N in ((2, 2 * 2 * 160), (4, 4 * 2 * 96), (3, 3 * 2 * 100)):
        for i in range(G):
            for j in range(G):
                out.append(lib.burst_attn_fill_zigzag_mask(i, j, G, N))
    for G, N in ((2, 2 * 300), (4, 4 * 256)):
        for i in range(G):
            for j in range(G):
                out.append(lib.burst_attn_fill_contiguous_mask(i, j, G, N))
                out.append(lib.burst_attn_fill_striped_mask(i, j, G, N))
    out.append(_custom_mask(lib, (10, 700), (0, 300), 150, 170, 1))     # pieces of different lengths on the two axes
    # many pieces (the block-striped split of block-wise sparse attention), also with piece lengths that are
    # not multiples of the tile sizes, a position stride inside the pieces, different piece counts per axis
    for G, N, N_blk in ((2, 1024, 256), (4, 1536, 384)):
        for i, j in ((0, 0), (1, 0), (0, G - 1), (G - 1, 1)):
            out.append(lib.burst_attn_fill_block_striped_mask(i, j, G, N, N_blk))
    out.append(_custom_mask(lib, (7, 307), (0, 450), 100, 150, 2, q_nseg=5, k_nseg=3))
    out.append(_custom_mask(lib, (0, 100), (50,), 40, 700, 1, q_nseg=9))
    out.append(_custom_mask(lib, (5, 900), (0,), 130, 400, 3))          # stride 3, mixed segment counts
    out.append(_custom_mask(lib, (40,), (0, 1000), 333, 200, 2))
    out.append(_custom_mask(lib, (0, 512), (0, 512), 256, 256, 1, causal=False))
    for window in (1, 40, 64, 150, 1000):   # sliding windows narrower than, equal to and wider than the tiles
        for m0 in (lib.burst_attn_fill_zigzag_mask(1, 0, 2, 2 * 2 * 160), lib.burst_attn_fill_zigzag_mask(0, 1, 2, 2 * 2 * 160),
                   lib.burst_attn_fill_zigzag_mask(2, 2, 4, 4 * 2 * 96), lib.burst_attn_fill_contiguous_mask(1, 0, 2, 600),
                   lib.burst_attn_fill_contiguous_mask(1, 1, 2, 600), lib.burst_attn_fill_striped_mask(3, 1, 4, 1024),
                   lib.burst_attn_fill_striped_mask(0, 2, 4, 1024), _custom_mask(lib, (5, 900), (0,), 130, 400, 3),
                   lib.burst_attn_fill_block_striped_mask(1, 0, 2, 1024, 256), lib.burst_attn_fill_block_striped_mask(0, 1, 2, 1024, 256),
                   lib.burst_attn_fill_block_striped_mask(3, 3, 4, 1536, 384),
                   _custom_mask(lib, (7, 307), (0, 450), 100, 150, 2, q_nseg=5, k_nseg=3)):
            m0.window = window
            out.append(m0)
    return out


def _vis(lib, m):
    return oc.visibility(hp.mask_positions(m, "q"), hp.mask_positions(m, "k"), m.mode == lib.BURST_MASK_CAUSAL, m.window)


def test_tile_classes_match_brute_force(lib):
    """Every (query block, key block) class the kernels can compute, by all three methods, against
    the visibility matrix of the oracle: skip <=> no visible pair, full <=> all pairs visible."""
    rng = np.random.default_rng(7)
    for m in _tile_logic_masks(lib):
        vis = _vis(lib, m)
        sq, sk = vis.shape
        blocks = [(q0, min(q0 + bq, sq), k0, min(k0 + bk, sk))
                  for bq, bk in ((64, 128), (256, 64), (32, 64), (64, 32))
                  for q0 in range(0, sq, bq) for k0 in range(0, sk, bk)]
        for q0, q1, k0, k1 in [blocks[t] for t in rng.permutation(len(blocks))[:120]]:
            sub = vis[q0:q1, k0:k1]
            want = 0 if not sub.any() else (1 if sub.all() else 2)
            got = [lib.burst_attn_tile_class(m, q0, q1, k0, k1, method) for method in (0, 1, 2)]
            assert got[0] == got[1] == got[2], (q0, q1, k0, k1, got)
            if m.window == 0:
                assert got[0] == want, (q0, q1, k0, k1, got, want)
            else:
                # the bounding ranges can be too coarse to see that a block is empty or whole when a
                # window meets position gaps (strides, two segments): "mixed" is then the safe verdict
                assert got[0] == want or got[0] == 2, (q0, q1, k0, k1, got, want)


def test_visible_tile_runs_match_brute_force(lib):
    """The closed-form runs of tiles a kernel walks hold exactly the tiles with a visible pair."""
    rng = np.random.default_rng(11)
    for m in _tile_logic_masks(lib):
        vis = _vis(lib, m)
        sq, sk = vis.shape
        for query_axis, tile, other_block in ((1, 64, 128), (1, 256, 128), (0, 64, 256), (0, 128, 256)):
            rows, other = (sq, sk) if query_axis else (sk, sq)
            for r0 in rng.permutation(np.arange(0, other, other_block))[:6]:
                r0, r1 = int(r0), int(min(r0 + other_block, other))
                sub = vis[:, r0:r1] if query_axis else vis[r0:r1, :].T     # [rows of the walked axis, other rows]
                n_tiles = -(-rows // tile)
                want = [bool(sub[t * tile:(t + 1) * tile].any()) for t in range(n_tiles)]
                runs = lib.burst_attn_visible_tile_runs(m, query_axis, tile, r0, r1)
                got = [False] * n_tiles
                prev_end = 0
                for start, length in runs:
                    if length:
                        assert start >= prev_end and start + length <= n_tiles
                        prev_end = start + length
                        for t in range(start, start + length):
                            got[t] = True
                if m.window == 0:
                    assert got == want, (query_axis, tile, r0, r1, runs)
                else:   # with a window the runs may hold tiles that turn out empty, never miss one
                    assert all(g or not w for g, w in zip(got, want)), (query_axis, tile, r0, r1, runs)
                    o_nseg, o_len = (m.k_nseg, m.k_seg_len) if query_axis else (m.q_nseg, m.q_seg_len)
                    w_nseg = m.q_nseg if query_axis else m.k_nseg
                    if o_nseg <= 2 and w_nseg <= 2 and not (o_nseg == 2 and r0 < o_len < r1) and m.window >= m.pos_stride:
                        # other rows inside one segment: only the tiles at the ends of a run can be empty
                        assert sum(got) <= sum(want) + 4, (query_axis, tile, r0, r1, runs, sum(want))


def test_pieces_must_be_in_position_order_and_not_overlap(lib):
    """The tile logic counts prefixes of rows below a position, which needs positions that grow with
    the local row: pieces out of order or overlapping are refused, and so are more than two pieces of
    fewer than 32 rows (a 32-row register tile may span two pieces, not three)."""
    INV, UNS = lib.BURST_ERR_INVALID_ARG, lib.BURST_ERR_UNSUPPORTED
    raw = lib.raw()
    cls = lambda m: raw.burst_attn_tile_class(C.byref(m), 0, 1, 0, 1, 0)
    assert cls(_custom_mask(lib, (700, 10), (0, 300), 150, 170, 1)) == INV          # second piece before the first
    assert cls(_custom_mask(lib, (0, 100), (0, 300), 150, 170, 1)) == INV           # pieces overlap
    assert cls(_custom_mask(lib, (0, 298), (0, 400), 150, 170, 2)) == INV           # ... because of the stride
    assert cls(_custom_mask(lib, (0, 299), (0, 400), 150, 170, 2)) >= 0
    assert cls(_custom_mask(lib, (0, 64), (0,), 16, 64, 1, q_nseg=3)) == UNS         # three pieces of 16 rows
    assert cls(_custom_mask(lib, (0, 64), (0,), 16, 64, 1, q_nseg=2)) >= 0
    assert cls(_custom_mask(lib, (0, 1 << 30), (0,), 64, 64, 1, q_nseg=4)) == UNS    # positions beyond 2^31
    assert lib.burst_attn_visible_pairs(_custom_mask(lib, (700, 10), (0, 300), 150, 170, 1)) == -1
    # the helper: N_blk must divide N and be a multiple of G
    m = lib.burst_mask_t()
    for args in ((0, 0, 4, 1024, 100), (0, 0, 4, 1024, 258), (0, 0, 4, 1024, 0), (4, 0, 4, 1024, 256)):
        assert raw.burst_attn_fill_block_striped_mask(*args, 1, C.byref(m)) == INV
    assert raw.burst_attn_fill_block_striped_mask(1, 2, 4, 1024, 256, 1, None) == INV


def test_tile_logic_rejects_bad_arguments(lib):
    m = lib.burst_attn_fill_zigzag_mask(1, 0, 2, 256)
    raw = lib.raw()
    assert raw.burst_attn_tile_class(None, 0, 1, 0, 1, 0) == lib.BURST_ERR_INVALID_ARG
    assert raw.burst_attn_tile_class(C.byref(m), 0, 0, 0, 1, 0) == lib.BURST_ERR_INVALID_ARG
    assert raw.burst_attn_tile_class(C.byref(m), 0, 1, 0, 1000, 0) == lib.BURST_ERR_INVALID_ARG
    assert raw.burst_attn_tile_class(C.byref(m), 0, 1, 0, 1, 9) == lib.BURST_ERR_INVALID_ARG
    out = (C.c_int32 * 4)()
    assert raw.burst_attn_visible_tile_runs(C.byref(m), 1, 48, 0, 1, C.byref(out)) == lib.BURST_ERR_UNSUPPORTED
    assert raw.burst_attn_visible_tile_runs(C.byref(m), 1, 64, 5, 5, C.byref(out)) == lib.BURST_ERR_INVALID_ARG


def test_block_pattern_slices_and_pair_counts(lib):
    """Host logic of the block-sparse benchmark workload: the per-step slice of a global block
    pattern, and the count of visible pairs under it, against the oracle's visibility matrix."""
    import bench
    from oracle import burst_oracle as oc
    from paper_2509_19836_amd import ring, workloads as wl
    G, N, R = 2, 2048, 256
    pattern = wl.block_sparse_pattern(N // R, 0.5, 11)
    assert pattern.shape == (8, 8) and pattern.diagonal().all() and 0 < pattern.sum() < 64
    for kind, window in (("zigzag", 0), ("causal", 0), ("causal", 300), ("full", 0)):
        for i in range(G):
            for j in range(G):
                m = ring.fill_mask(kind, i, j, G, N, window)
                pos_q, pos_k = ring.mask_positions(m, "q"), ring.mask_positions(m, "k")
                bm = wl.local_block_mask(pattern, pos_q, pos_k, R)
                # brute force: the pattern entry of the global blocks of each (q, k) pair
                want = pattern[np.ix_(pos_q // R, pos_k // R)].astype(bool)
                vis = oc.visibility(pos_q, pos_k, kind != "full", window)
                masked = oc.apply_block_mask(vis, bm, R, R)
                assert np.array_equal(masked, vis & want)
                assert bench.block_masked_pairs(bm, pos_q, pos_k, R, kind != "full", window) == int(masked.sum())
    with pytest.raises(ValueError):   # striped rows do not form blocks of consecutive tokens
        m = ring.fill_mask("striped", 0, 1, G, N)
        wl.local_block_mask(pattern, ring.mask_positions(m, "q"), ring.mask_positions(m, "k"), R)


def test_lm_head_arguments_are_checked_on_the_host(lib):
    """Validation of the fused LM head + loss call: nothing here reaches a launch; the pointers are
    made-up numbers that are never dereferenced."""
    raw = lib.raw()
    INV, UNS = lib.BURST_ERR_INVALID_ARG, lib.BURST_ERR_UNSUPPORTED
    ok = lib.lm_head_shape(1000, 512, 3000, 256)
    need = lib.burst_lm_head_workspace_bytes(ok)
    v_pad = 3072
    assert need == 256 * v_pad * 4 + 256 * v_pad * 2 + (v_pad // 128) * 256 * 8 + 512 * 256 * 2
    for bad in (lib.lm_head_shape(-1, 512, 3000, 256), lib.lm_head_shape(10, 512, 0, 256),
                lib.lm_head_shape(10, 512, 3000, 100), lib.lm_head_shape(10, 512, 3000, 0),
                lib.lm_head_shape(10, 0, 3000, 256), lib.lm_head_shape(10, 512, 3000, 256, float("inf"))):
        assert raw.burst_lm_head_workspace_bytes(C.byref(bad)) == -1

    def call(shape=ok, h=0x10000, ld_h=512, w=0x20000, ld_w=512, y=0x30000, loss=0x40000, lse=None, dh=0x50000,
             dh_dtype=1, ld_dh=512, dw=0x60000, ld_dw=512, ws=0x70000, ws_bytes=need):
        return raw.burst_lm_head_loss(C.byref(shape) if shape is not None else None, h, ld_h, w, ld_w, y, loss, lse, dh,
                                      dh_dtype, ld_dh, dw, ld_dw, 0, ws, ws_bytes, None)
    assert call(shape=None) == INV
    assert call(shape=lib.lm_head_shape(1000, 500, 3000, 256)) == UNS      # d not a multiple of 256
    assert call(shape=lib.lm_head_shape(1000, 512, 1 << 23, 256)) == UNS   # vocabulary beyond the 32-bit tile offsets
    assert call(h=None) == INV and call(w=None) == INV and call(y=None) == INV and call(loss=None) == INV
    assert call(h=0x10008) == INV                                          # misaligned
    assert call(ld_h=504) == INV and call(ld_w=511) == INV                 # leading dimension below d / not a multiple of 8
    assert call(dh_dtype=7) == INV and call(ld_dh=256) == INV and call(ld_dw=510) == INV
    assert call(ws=None) == INV and call(ws=0x70010) == INV and call(ws_bytes=need - 1) == INV


def test_lm_head_noalloc_entry_point_checks_shape_and_scratch_limit_on_the_host(lib):
    """burst_lm_head_loss_noalloc refuses, before touching any GPU, an invalid shape and a shape whose
    workspace exceeds the library's built-in scratch array; the pointers are never dereferenced."""
    raw = lib.raw()
    limit = lib.burst_lm_head_static_scratch_bytes()
    assert limit == 64 << 20

    def call(shape):
        return raw.burst_lm_head_loss_noalloc(C.byref(shape) if shape is not None else None, 0x10000, 512, 0x20000, 512,
                                              0x30000, 0x40000, None, 0x50000, 1, 512, 0x60000, 512, 0, None)
    assert call(None) == lib.BURST_ERR_INVALID_ARG
    assert call(lib.lm_head_shape(1000, 500, 3000, 256)) == lib.BURST_ERR_UNSUPPORTED
    fits = lib.lm_head_shape(1000, 4096, 32000, 256)
    too_big = lib.lm_head_shape(1000, 4096, 32000, 512)
    assert lib.burst_lm_head_workspace_bytes(fits) <= limit < lib.burst_lm_head_workspace_bytes(too_big)
    assert call(too_big) == lib.BURST_ERR_SCRATCH
    assert "scratch" in lib.burst_attn_status_string(lib.BURST_ERR_SCRATCH)


def _range_positions(rg, stride):
    return np.concatenate([rg["pos0"] + s * rg["period"] + np.arange(rg["seg_len"], dtype=np.int64) * stride
                           for s in range(rg["nseg"])])


@pytest.mark.parametrize("chunk_rows", [256, 1024])
def test_backward_chunk_plan_covers_the_axis_with_the_same_positions(lib, chunk_rows):
    """The ranges the backward launcher cuts a streamed axis into (host logic, no GPU): they tile the axis in
    order, every range is a chunk the mask descriptor expresses (inside one piece, or whole pieces), its rows
    have the positions the step's mask gives them, and with a block mask every range starts on a block row."""
    G = 4
    assert lib.burst_attn_set_chunk_rows(chunk_rows) == chunk_rows
    try:
        cases = [("causal", 4 * 6000, 0), ("zigzag", 4 * 2 * 1536, 0), ("zigzag", 4 * 2 * 1100, 0), ("striped", 4 * 5000, 0),
                 ("block_striped", 4 * 4096, 512), ("block_striped", 4 * 3072, 1536), ("block_striped", 4 * 8192, 8192)]
        for kind, N, N_blk in cases:
            m = hp.fill_mask(lib, kind, 1, 2, G, N, 0, N_blk)
            for axis, side in ((1, "q"), (0, "k")):
                pos = hp.mask_positions(m, side)
                plan = lib.burst_attn_chunk_plan(m, axis)
                assert plan[0]["r0"] == 0 and plan[-1]["r1"] == pos.size, (kind, N, plan)
                if pos.size > 2 * chunk_rows:
                    assert len(plan) > 1, (kind, N, chunk_rows)
                for a, b in zip(plan, plan[1:]):
                    assert a["r1"] == b["r0"]
                for rg in plan:
                    assert rg["r1"] - rg["r0"] == rg["nseg"] * rg["seg_len"] > 0
                    assert (_range_positions(rg, m.pos_stride) == pos[rg["r0"]:rg["r1"]]).all(), (kind, N, rg)
        # a block mask: ranges start on block rows, the mask pointer moves by whole block rows (query axis) or
        # block columns (key axis); blocks that the ranges would cut switch the chunking off
        m = hp.fill_mask(lib, "zigzag", 1, 2, G, 4 * 2 * 2048)
        m.block_mask = 1 << 20   # an address the host never dereferences
        m.q_block_rows, m.k_block_rows, m.block_pitch = 256, 128, 64
        for rg in lib.burst_attn_chunk_plan(m, 1):
            assert rg["r0"] % 256 == 0 and rg["blk_offset"] == (rg["r0"] // 256) * 64
        for rg in lib.burst_attn_chunk_plan(m, 0):
            assert rg["r0"] % 128 == 0 and rg["blk_offset"] == rg["r0"] // 128
        m.q_block_rows = 768   # 768 does not divide the range length: one launch
        assert len(lib.burst_attn_chunk_plan(m, 1)) == 1
        assert len(lib.burst_attn_chunk_plan(hp.fill_mask(lib, "causal", 1, 2, G, 4 * 2 * chunk_rows), 1)) == 1
    finally:
        lib.burst_attn_set_chunk_rows(32768)
