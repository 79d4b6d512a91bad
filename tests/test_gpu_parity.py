"""GPU parity: the HIP decode path against the fp64 CPU oracle, through the C ABI.

Tolerances (from the benchmark spec): max-abs 1e-3 per fp32 channel value, +-1 LSB after
uint8 conversion, bit-exact for the pack / dequantise / gather path.
"""
import ctypes as C

import numpy as np
import pytest

from oracle import oracle
from paper_2306_16699_amd import rinr, synth
from paper_2306_16699_amd.synth import Layer, Model

pytestmark = pytest.mark.gpu

TOL = 1e-3
TIGHT = 2e-5          # what the default and the fp32 kernels are held to on top of TOL (measured: 3e-7 .. 3e-6)
UNCHECKED = rinr.FLAG_FP16_UNCHECKED
# every way to ask for a kernel family: the default, fp32 MFMA, the two reduced-precision modes as the library grants
# them (only where the store's a-priori error bound allows, else the default kernels run), and the same two forced
MODES = (0, rinr.FLAG_FP32_MFMA, rinr.FLAG_FP16_ACT, rinr.FLAG_FP16_ALL, rinr.FLAG_FP16_ACT | UNCHECKED, rinr.FLAG_FP16_ALL | UNCHECKED)


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available()
    rinr.lib()          # fail loudly if the HIP library is not built
    return t


def ids_dev(torch, ids):
    return torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int64)).cuda()


def image_like(models):
    """Parity-only variant: output weights x10 and bias +0.5 so values span [0, 1] and both clamp edges."""
    out = []
    for m in models:
        last = m.layers[-1]
        assert last.bits == 0
        nl = Layer(last.n_in, last.n_out, 0, 0.0, 0, (last.weights * np.float32(10)).astype(np.float32), last.keep,
                   (last.bias + np.float32(0.5)).astype(np.float32))
        out.append(Model(m.layers[:-1] + [nl]))
    return out


WORST = {}       # largest unclamped error seen per mode, printed at the end of the run


def check_workload(torch, w, models=None, tile=0, u8=False, **launch):
    """Every kernel family against the oracle at the one tolerance; `launch` forces a launch shape."""
    models = models if models is not None else w.models
    st = rinr.Store(rinr.pack(models, w.w0, w.coord_lo, w.coord_hi), fp32_tile_rows=tile)
    ids = ids_dev(torch, w.image_ids)
    bounds = st.error_bounds()
    ref_nc = oracle.decode(models, w.image_ids, w.H, w.W, w.w0, w.coord_lo, w.coord_hi, clamp=False)
    ref, ref8 = oracle.decode(models, w.image_ids, w.H, w.W, w.w0, w.coord_lo, w.coord_hi, want_u8=True)
    worst = 0.0
    for mode in MODES:
        got_nc = st.decode_batch_ex(ids, w.H, w.W, rinr.OUT_F32, mode | rinr.FLAG_NO_CLAMP, **launch).cpu().numpy().astype(np.float64)
        ran = st.last_launch_info()["kernels"]
        # a reduced-precision family runs exactly where it is forced or its bound allows it
        if mode & rinr.FLAG_FP16_ALL:
            want = 3 if (mode & UNCHECKED or bounds[1] <= 9.5e-4) else (2 if bounds[0] <= 9.5e-4 else 0)
        elif mode & rinr.FLAG_FP16_ACT:
            want = 2 if (mode & UNCHECKED or bounds[0] <= 9.5e-4) else 0
        else:
            want = 1 if mode & rinr.FLAG_FP32_MFMA else 0
        assert ran == rinr.FAMILIES[want], (mode, ran, bounds)
        err_nc = np.abs(got_nc - ref_nc).max()
        WORST[mode] = max(WORST.get(mode, 0.0), err_nc)
        if want >= 2:
            assert err_nc <= bounds[want - 2] + 1e-6, (mode, err_nc, bounds)   # the worst-case bound is one
        if mode & UNCHECKED and bounds[want - 2] > 9.5e-4:
            # forced past its bound, a reduced-precision family promises nothing: its error is reported at the end of the
            # run and asserted on the benchmark workloads at full size
            assert np.isfinite(got_nc).all()
            continue
        assert err_nc <= TOL, f"mode {mode}: unclamped max-abs {err_nc}"
        if want <= 1:
            # the full-precision families sit orders of magnitude inside the tolerance; holding them there makes a lost
            # low-half term of a contraction (about 1e-4) visible, which the tolerance itself would let pass
            assert err_nc <= TIGHT, f"mode {mode}: unclamped max-abs {err_nc} (full-precision families are held to {TIGHT})"
        worst = max(worst, err_nc)
        got = st.decode_batch_ex(ids, w.H, w.W, rinr.OUT_F32, mode, **launch).cpu().numpy()
        assert got.min() >= 0.0 and got.max() <= 1.0
        assert np.abs(got.astype(np.float64) - ref).max() <= TOL
        if mode == 0 and not launch:
            assert np.array_equal(st.decode_batch(ids, w.H, w.W).cpu().numpy(), got)   # plain entry point = default mode
        if u8:
            g32, g8 = st.decode_batch_ex(ids, w.H, w.W, rinr.OUT_F32_AND_U8, mode, **launch)
            assert np.array_equal(g32.cpu().numpy(), got)               # same kernel, same bits
            g8 = g8.cpu().numpy()
            assert np.abs(g8.astype(np.int32) - ref8.astype(np.int32)).max() <= 1
            only8 = st.decode_batch_ex(ids, w.H, w.W, rinr.OUT_U8, mode, **launch).cpu().numpy()
            assert np.array_equal(only8, g8)
            # the uint8 is the rounding of the fp32 the kernel produced
            assert np.array_equal(g8, np.rint(255.0 * got.astype(np.float32)).astype(np.uint8))
    assert st.status() == 0
    st.close()
    return worst


# ---- dequantise / expand stage: bit-exact against the oracle ------------------------------------------------
@pytest.mark.parametrize("tile", [16, 32])
def test_dequant_bit_exact(torch, tile):
    rng = np.random.default_rng(7)
    models = []
    for width in (1, 7, 16, 20, 24, 32, 33, 40, 48, 57, 64):
        for kp in (None, 0.0, 0.35, 1.0):
            dims = [2] + [width] * int(rng.integers(1, 5)) + [3]
            layers = []
            for l in range(len(dims) - 1):
                n_in, n_out = dims[l], dims[l + 1]
                bits = int(rng.choice([0, 2, 3, 4, 5, 6, 7, 8, 16]))
                if bits == 0:
                    wt = rng.uniform(-0.5, 0.5, (n_out, n_in)).astype(np.float32)
                    scale, zp = 0.0, 0
                else:
                    wt = rng.integers(0, 1 << bits, (n_out, n_in)).astype(np.uint8 if bits <= 8 else np.uint16)
                    scale, zp = float(np.float32(rng.uniform(1e-4, 1e-2))), int(rng.integers(0, 1 << bits))
                keep = None if kp is None else (rng.uniform(size=(n_out, n_in)) < kp).astype(np.uint8)
                layers.append(Layer(n_in, n_out, bits, scale, zp, wt, keep, rng.uniform(-.1, .1, n_out).astype(np.float32)))
            models.append(Model(layers))
    st = rinr.Store(rinr.pack(models), fp32_tile_rows=tile)
    for mi, m in enumerate(models):
        for li, ly in enumerate(m.layers):
            wd, bd = st.debug_dequant(mi, li, ly.n_in, ly.n_out)
            want = oracle.dequant(ly).astype(np.float32)       # exact: the doubles hold fp32 values
            got = wd.cpu().numpy()
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (mi, li, ly.bits, ly.n_in, ly.n_out)
            assert np.array_equal(bd.cpu().numpy(), ly.bias)
            if tile == 32:
                check_split_blocks(st, mi, li, len(m.layers), ly, want)
    st.close()


def check_split_blocks(st, mi, li, n_layers, ly, want):
    """The default kernels' fp16 operand blocks, element by element, against the oracle's dequantised weights `want`
    (fp32): a 2..8-bit hidden layer is held as the integers code - zp, with the scale kept apart, and scale * integer
    must be the oracle's value bit for bit; every other layer is held as hi = fp16(w), lo = fp16(w - hi), both
    determined by the oracle's value; with fp16 weights the one block is fp16(w)."""
    hi, lo, b, sc = (t.cpu().numpy() for t in st.debug_dequant_split(mi, li, ly.n_in, ly.n_out))
    hidden = 0 < li < n_layers - 1
    if hidden and 2 <= ly.bits <= 8:
        assert np.array_equal(hi, np.rint(hi)) and np.abs(hi).max() <= 255 and not lo.any()
        assert np.float32(sc[0]) == np.float32(ly.scale)
        assert np.array_equal((np.float32(sc[0]) * hi.astype(np.float32)).view(np.uint32), want.view(np.uint32)), (mi, li)
        assert np.allclose(b.astype(np.float64) * float(sc[0]), ly.bias, rtol=3e-7, atol=0)       # the bias tile holds bias / scale
    else:
        h16 = want.astype(np.float16).astype(np.float32)
        assert sc[0] == 1.0
        assert np.array_equal(hi.view(np.uint32), h16.view(np.uint32)), (mi, li, ly.bits)
        assert np.array_equal(lo.view(np.uint32), (want - h16).astype(np.float16).astype(np.float32).view(np.uint32)), (mi, li, ly.bits)
        assert np.array_equal(b, ly.bias)
    if hidden:
        hi16, lo16, b16, sc16 = (t.cpu().numpy() for t in st.debug_dequant_split(mi, li, ly.n_in, ly.n_out, fp16_weights=True))
        assert np.array_equal(hi16.view(np.uint32), want.astype(np.float16).astype(np.float32).view(np.uint32)) and not lo16.any()
        assert sc16[0] == 1.0 and np.array_equal(b16, ly.bias)


# ---- gather: constant-colour models make the id -> plane map exact -------------------------------------------
def test_gather_exact_with_repeats_and_bad_ids(torch):
    n_models = 300
    rng = np.random.default_rng(1)
    models = []
    for i in range(n_models):
        width = [8, 24, 40, 64][i % 4]
        col = np.array([(i % 256) / 255.0, ((i * 7) % 256) / 255.0, ((i * 13) % 256) / 255.0], np.float32)
        models.append(Model([Layer(2, width, 0, 0, 0, np.zeros((width, 2), np.float32), None, np.zeros(width, np.float32)),
                             Layer(width, 3, 0, 0, 0, np.zeros((3, width), np.float32), None, col)]))
    st = rinr.Store(rinr.pack(models))
    ids = rng.integers(0, n_models, 500)
    ids[[3, 77, 78, 400]] = [-1, n_models, 2 ** 40, -2 ** 62]
    H, W = 5, 13
    f32, u8 = st.decode_batch_ex(ids_dev(torch, ids), H, W, rinr.OUT_F32_AND_U8)
    f32, u8 = f32.cpu().numpy(), u8.cpu().numpy()
    for s, i in enumerate(ids):
        if 0 <= i < n_models:
            want = models[i].layers[1].bias
            assert np.array_equal(f32[s], np.broadcast_to(want[:, None, None], (3, H, W))), (s, i)
            assert np.array_equal(u8[s, :, 0, 0], np.array([i % 256, (i * 7) % 256, (i * 13) % 256], np.uint8))
        else:
            assert not f32[s].any() and not u8[s].any()
    assert st.status() == 4
    st.decode_batch(ids_dev(torch, ids[:100]), H, W)
    assert st.status() == 7                                  # sticky: 4 + the 3 bad ids among the first 100
    st.close()


# ---- the five workloads at sizes the oracle finishes in seconds; several tiles and a ragged tail -----------
@pytest.mark.parametrize("k,n,H,W", [(1, 64, 32, 32), (2, 96, 32, 32), (3, 24, 64, 64), (4, 6, 75, 53), (4, 4, 224, 224)])
def test_parity_uniform_workloads(torch, k, n, H, W):
    w = synth.workload(k, n_images=n, H=H, W=W)
    check_workload(torch, w, u8=(k == 4))
    check_workload(torch, w, models=image_like(w.models), u8=True)


@pytest.mark.parametrize("k,n,H,W", [(2, 32, 32, 32), (4, 4, 75, 53)])
def test_parity_tile16_variant(torch, k, n, H, W):
    w = synth.workload(k, n_images=n, H=H, W=W)
    check_workload(torch, w, models=image_like(w.models), tile=16, u8=True)


@pytest.mark.parametrize("threads,blocks_per_cu,any_min", [(256, 0, 0), (512, 3, 0), (768, 16, 0), (0, 1, 1), (0, 0, 1 << 20)])
def test_parity_under_other_launch_shapes(torch, threads, blocks_per_cu, any_min):
    """The planner picks threads per workgroup, workgroups per slot and, for stores of mixed width, one grid or class by
    class from the image size: here they are forced through the decode options, on a uniform and on a ragged workload."""
    shape = dict(threads=threads, blocks_per_cu=blocks_per_cu, one_grid_min_tiles=any_min)
    check_workload(torch, synth.workload(3, n_images=6, H=70, W=83), **shape)
    w = synth.workload(5, n_images=48, pool=300, H=72, W=65)
    check_workload(torch, w, models=image_like(w.models), u8=True, **shape)


def test_parity_ragged_pool(torch):
    w = synth.workload(5, n_images=64, pool=400, H=40, W=37)
    assert len({(m.width, m.n_sine_layers) for m in w.models}) == 20
    check_workload(torch, w)
    check_workload(torch, w, models=image_like(w.models), u8=True)


def test_all_layers_coded_and_paper_coordinate_range(torch):
    ms = synth._uniform_models(11, 8, 32, 4, (6, 8), 0.5, code_all=True)
    w = synth.Workload("all-coded", ms, np.arange(8)[::-1].copy(), 19, 23, False, 30.0, 0.0, 1.0)
    check_workload(torch, w)


def test_paper_shaped_models(torch):
    """Sec. VI-A shapes: 10 layers x 40 hidden, 10 x 32, 3 x 15; 16-bit codes (Fig. 3); a tapered shape (Sec. V-A)."""
    ids = np.arange(3)
    ms = (synth.make_models(21, ids[:1], 40, 9, [0] + [8] * 8 + [0], 0.75)
          + synth.make_models(21, ids[1:2], 32, 9, [0] + [16] * 8 + [0], 0.8)
          + synth.make_models(21, ids[2:3], 15, 2, [0, 8, 0], 0.85))
    ms += synth.make_models(22, np.arange(1), 0, 5, [0, 8, 8, 8, 8, 0], 0.8, widths=[16, 32, 48, 32, 16])
    w = synth.Workload("paper-shaped", ms, np.array([3, 0, 1, 2, 3]), 33, 31, False)
    check_workload(torch, w)
    check_workload(torch, w, models=image_like(ms), u8=True)


@pytest.mark.parametrize("width", [5, 8, 9, 40, 41, 50, 56])
def test_widths_around_half_a_row_tile(torch, width):
    """Widths just below, at and above half a 16-row tile and a full one (padding rows of every amount)."""
    ms = synth._uniform_models(31 + width, 6, width, 3, (6, 8), 0.6) + synth._uniform_models(57 + width, 2, width, 2, None, None)
    w = synth.Workload(f"width {width}", ms, np.array([7, 0, 3, 5, 6, 1]), 21, 19, False)
    check_workload(torch, w)
    check_workload(torch, w, models=image_like(ms), u8=True)


# ---- degenerate sizes ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("H,W", [(1, 1), (1, 63), (64, 1), (1, 65), (8, 8), (9, 7), (127, 1)])
def test_small_and_ragged_grids(torch, H, W):
    w = synth.workload(2, n_images=5, H=H, W=W)
    check_workload(torch, w, models=image_like(w.models), u8=True)


@pytest.mark.parametrize("H,W", [(1201, 1999), (1024, 2048)])
def test_few_large_images(torch, H, W):
    """Millions of pixels per image: many workgroups per slot, pixel indices far beyond one tile row, W a power of
    two and not (the row/column split of a pixel index is a multiply-high by a constant made from W)."""
    w = synth.workload(1, n_images=2, H=H, W=W)
    st = rinr.Store(rinr.pack(w.models, w.w0, w.coord_lo, w.coord_hi))
    ids = ids_dev(torch, w.image_ids)
    ref = oracle.decode(w.models, w.image_ids, H, W, w.w0, w.coord_lo, w.coord_hi, clamp=False)
    for mode in (0, rinr.FLAG_FP32_MFMA, rinr.FLAG_FP16_ALL):
        got = st.decode_batch_ex(ids, H, W, rinr.OUT_F32, mode | rinr.FLAG_NO_CLAMP).cpu().numpy()
        assert np.abs(got - ref).max() <= TOL, mode
        assert st.last_launch_info()["workgroups"] > 2
    st.close()


def test_resolution_free_decode(torch):
    """Same store decoded at several resolutions (Sec. III-B): nested pixel-centre grids agree."""
    w = synth.workload(3, n_images=3, H=10, W=12)
    st = rinr.Store(rinr.pack(image_like(w.models)))
    ids = ids_dev(torch, w.image_ids)
    a = st.decode_batch(ids, 10, 12).cpu().numpy()
    b = st.decode_batch(ids, 30, 36).cpu().numpy()
    assert np.abs(a - b[:, :, 1::3, 1::3]).max() < 2e-4
    st.close()


def test_duplicates_bit_identical_and_n0(torch):
    w = synth.workload(3, n_images=4, H=17, W=9)
    st = rinr.Store(rinr.pack(w.models))
    out = st.decode_batch(ids_dev(torch, [2, 2, 0, 2]), 17, 9).cpu().numpy()
    assert np.array_equal(out[0], out[1]) and np.array_equal(out[0], out[3])
    empty = st.decode_batch(torch.zeros(0, dtype=torch.int64, device="cuda"), 17, 9)
    assert tuple(empty.shape) == (0, 3, 17, 9)
    assert st.last_launch_info()["launches"] == 0
    st.close()


def test_empty_store_zero_fills_and_counts(torch):
    st = rinr.Store(rinr.pack([]))
    assert st.info() == (0, 0, 0)
    out = torch.full((3, 3, 5, 7), 9.0, device="cuda")
    st.decode_batch(ids_dev(torch, [0, 1, -5]), 5, 7, out=out)
    assert st.status() == 3 and not out.cpu().numpy().any()
    st.close()


def test_decode_on_side_stream_and_preallocated_out(torch):
    w = synth.workload(2, n_images=16)
    st = rinr.Store(rinr.pack(w.models))
    ids = ids_dev(torch, w.image_ids)
    ref = st.decode_batch(ids, 32, 32).cpu().numpy()
    out = torch.full((16, 3, 32, 32), -7.0, device="cuda")
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        st.decode_batch(ids, 32, 32, out=out)
    s.synchronize()
    assert np.array_equal(out.cpu().numpy(), ref)
    st.close()


def test_decode_replayed_from_a_captured_graph(torch):
    """A decode call enqueues one kernel and nothing else, so it can be captured once and replayed with other
    ids in the same buffers (tight serving loops); every replay is checked against an eager call."""
    w = synth.workload(5, n_images=24, pool=64, H=40, W=36)          # ragged store: the all-class kernel
    st = rinr.Store(rinr.pack(w.models))
    rng = np.random.default_rng(5)
    ids = ids_dev(torch, w.image_ids)
    out = torch.empty((24, 3, 40, 36), device="cuda")
    out8 = torch.empty((24, 3, 40, 36), dtype=torch.uint8, device="cuda")
    st.decode_batch_ex(ids, 40, 36, rinr.OUT_F32_AND_U8, out=out, out_u8=out8)     # plans the launch before capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        st.decode_batch_ex(ids, 40, 36, rinr.OUT_F32_AND_U8, out=out, out_u8=out8)
    for _ in range(3):
        ids.copy_(torch.from_numpy(rng.integers(0, 64, 24).astype(np.int64)))
        out.fill_(-3.0)
        out8.fill_(7)
        g.replay()
        torch.cuda.synchronize()
        ref, ref8 = st.decode_batch_ex(ids, 40, 36, rinr.OUT_F32_AND_U8)
        torch.cuda.synchronize()
        assert torch.equal(out, ref) and torch.equal(out8, ref8)
    assert st.status() == 0
    del g
    st.close()


def test_store_open_validates_on_device_copy(torch):
    w = synth.workload(2, n_images=3)
    blob = rinr.pack(w.models)
    st = rinr.Store(blob, validate_on_device=True)
    assert st.info() == (3, 32, 5)
    st.close()
    bad = blob.copy(); bad[0] ^= 0xFF
    with pytest.raises(rinr.RinrError) as e:
        rinr.Store(bad, validate_on_device=True)
    assert e.value.code == rinr.E_FORMAT


def test_models_too_deep_for_lds_are_streamed(torch):
    """Everything the packer accepts decodes, in every kernel family.  A model whose expanded weights and packed
    record do not fit the 160 KB of on-chip memory is decoded with its layers streamed through it in groups: same
    results, slower.  Up to the format's limits at once (16 linear layers of width 64), dense and sparse, 8-bit and
    raw fp32 hidden layers, next to shallow models of the same store that stay resident."""
    deep8 = synth.make_models(3, np.arange(2), 64, 12, [0] + [8] * 11 + [0], 0.5)          # fits as fp16 blocks, not as fp32
    dense = synth.make_models(4, np.arange(2), 64, 15, [0] + [8] * 14 + [0], 0.9)         # 16 layers, dense records
    sparse = synth.make_models(4, np.arange(2), 64, 15, [0] + [8] * 14 + [0], 0.1)
    raw = synth.make_models(3, np.arange(1), 64, 12, [0] * 13, 0.5)                       # raw fp32 hidden layers: two blocks each
    narrow = synth.make_models(6, np.arange(2), 40, 15, [0] + [8, 0, 16] * 4 + [8, 8] + [0], 0.7)   # mixed kinds, width class 3
    shallow = synth.make_models(5, np.arange(2), 64, 3, [0, 8, 8, 0], 0.5) + synth.make_models(5, np.arange(1), 24, 2, [0, 8, 0], 0.5)
    for name, models, streamed_default, streamed_fp32 in (("deep8", deep8, False, True), ("dense16", dense, True, True),
                                                          ("sparse16", sparse, False, True), ("raw13", raw, True, True),
                                                          ("mixed", dense + shallow + raw + narrow, True, True)):
        st = rinr.Store(rinr.pack(models))
        assert st.info()[0] == len(models)
        order = np.arange(len(models))[::-1].copy()
        ids = ids_dev(torch, order)
        H, W = 21, 37                                              # 13 tiles: several rounds of four wavefronts and a ragged one
        ref = oracle.decode(models, order, H, W, clamp=False)
        ref8 = oracle.decode(models, order, H, W, want_u8=True)[1]
        for mode in MODES:
            got = st.decode_batch_ex(ids, H, W, rinr.OUT_F32, mode | rinr.FLAG_NO_CLAMP).cpu().numpy()
            info = st.last_launch_info()
            if mode == 0:
                assert info["streamed"] == streamed_default, (name, info)
            if mode == rinr.FLAG_FP32_MFMA:
                assert info["streamed"] == streamed_fp32, (name, info)
            err = np.abs(got - ref).max()
            if mode & UNCHECKED:                                   # forced reduced precision has no bound at this depth
                assert np.isfinite(got).all()
                continue
            assert err <= TOL, (name, mode, err)
            u8 = st.decode_batch_ex(ids, H, W, rinr.OUT_U8, mode).cpu().numpy()
            assert np.abs(u8.astype(np.int32) - ref8.astype(np.int32)).max() <= 1, (name, mode)
        assert st.status() == 0
        st.close()


def test_streamed_decode_equals_resident_decode_bit_for_bit(torch):
    """The streamed kernels run the same arithmetic in the same order as the resident ones.  A store opened with a small
    on-chip budget streams models that another handle on the same blob keeps resident: same bytes out, for groups of one
    layer up to several, in every family, with augmentation and both outputs; and the resident models of a store that
    also holds a streamed one are not changed by it."""
    w = synth.workload(5, n_images=40, pool=120, H=30, W=41)
    ms = image_like(w.models) + synth.make_models(8, np.arange(2), 48, 4, [0, 0, 16, 8, 0], 0.7)     # raw and 16-bit hidden layers too
    blob = rinr.pack(ms)
    ids = ids_dev(torch, np.concatenate([w.image_ids, [120, 121]]))
    n = int(ids.numel())
    aff = torch.from_numpy(np.random.default_rng(3).uniform(-1, 1, (n, 6)).astype(np.float32)).cuda()
    big = rinr.Store(blob)
    for budget in (20 * 1024, 36 * 1024, 64 * 1024):
        small = rinr.Store(blob, lds_budget=budget)
        for mode in MODES:
            a32, a8 = big.decode_batch_ex(ids, 30, 41, rinr.OUT_F32_AND_U8, mode, affine=aff)
            assert not big.last_launch_info()["streamed"]
            b32, b8 = small.decode_batch_ex(ids, 30, 41, rinr.OUT_F32_AND_U8, mode, affine=aff)
            assert small.last_launch_info()["streamed"], (budget, mode)
            assert torch.equal(a32, b32) and torch.equal(a8, b8), (budget, mode)
        assert small.status() == 0
        small.close()
    big.close()
    with pytest.raises(rinr.RinrError) as e:
        rinr.Store(blob, lds_budget=1000)
    assert e.value.code == rinr.E_ARG


@pytest.mark.parametrize("width", [12, 32, 40, 48, 64])
def test_every_term_of_the_output_layer_arrives(torch, width):
    """A model whose first and hidden layers have zero weights: the last sine layer's outputs are the constants
    sin(w0 b), so the image is one colour that the CPU gives in closed form, sum_i W[c][i] sin(w0 b_i) + b_c, to 1e-6,
    in every kernel family, resident and streamed.  The split-precision kernels add the output layer up from several
    matrix instructions per accumulator (high and low halves of the weights, full-depth and half-depth steps); each
    contributes 1e-4 or more here, so one that is lost (two instructions of different depth too close together on one
    accumulator lose the first one's result) cannot hide below the 1e-3 tolerance."""
    rng = np.random.default_rng(width)
    b1 = rng.uniform(-.1, .1, width).astype(np.float32)
    Wo = rng.uniform(-1, 1, (3, width)).astype(np.float32)
    bo = rng.uniform(0.2, 0.8, 3).astype(np.float32)
    m = Model([Layer(2, width, 0, 0, 0, np.zeros((width, 2), np.float32), None, rng.uniform(-.1, .1, width).astype(np.float32)),
               Layer(width, width, 8, 1e-3, 128, np.full((width, width), 128, np.uint8), None, b1),
               Layer(width, 3, 0, 0, 0, Wo, None, bo)])
    h = np.sin(30.0 * b1.astype(np.float64))
    h16 = h.astype(np.float32).astype(np.float16).astype(np.float64)          # one fp16 value per activation
    W64 = Wo.astype(np.float64)
    Wh = Wo.astype(np.float16).astype(np.float64)
    assert np.abs((W64 - Wh)[:, :32] @ h[:32]).max() > 5e-5                     # the low halves' term is far above the check below
    exact = W64 @ h + bo
    exact16 = W64 @ h16 + bo
    assert np.abs(oracle.decode([m], [0], 3, 5, clamp=False)[0, :, 0, 0] - exact).max() < 1e-12
    ids = ids_dev(torch, [0, 0, 0])
    blob = rinr.pack([m])
    for budget in (0, 20 * 1024):
        st = rinr.Store(blob, lds_budget=budget)
        for mode in MODES:
            got = st.decode_batch_ex(ids, 9, 15, rinr.OUT_F32, mode | rinr.FLAG_NO_CLAMP).cpu().numpy().astype(np.float64)
            fam = st.last_launch_info()["kernels"]
            want = exact16 if fam in rinr.FAMILIES[2:] else exact
            err = np.abs(got - want[None, :, None, None]).max()
            assert err < 1e-5, (width, budget, mode, fam, err)
        st.close()


def test_reduced_precision_is_granted_by_the_error_bound(torch):
    """RINR_FLAG_FP16_ACT / _ALL run their kernels only on stores whose worst-case error bound is below the tolerance;
    elsewhere the default kernels serve the call and the result is the default's, bit for bit."""
    # the paper's small-image shape (Sec. VI-A: 15 hidden units, one hidden layer): the bound certifies it
    small = synth.make_models(9, np.arange(6), 15, 2, [0, 8, 0], 0.85)
    st = rinr.Store(rinr.pack(small, 30.0, 0.0, 1.0))
    b = st.error_bounds()
    assert b[0] <= 9.5e-4 and b[1] >= b[0]
    ids = ids_dev(torch, np.arange(6))
    ref = oracle.decode(small, np.arange(6), 32, 32, 30.0, 0.0, 1.0, clamp=False)
    d = st.decode_batch_ex(ids, 32, 32, rinr.OUT_F32, rinr.FLAG_NO_CLAMP)
    g = st.decode_batch_ex(ids, 32, 32, rinr.OUT_F32, rinr.FLAG_NO_CLAMP | rinr.FLAG_FP16_ACT)
    assert st.last_launch_info()["kernels"] == rinr.FAMILIES[2]
    assert not torch.equal(d, g)                                   # another kernel did run
    assert np.abs(g.cpu().numpy() - ref).max() <= b[0] <= TOL
    st.close()
    # a deep model: far beyond any bound, the flags change nothing
    w = synth.workload(4, n_images=2, H=40, W=40)
    st = rinr.Store(rinr.pack(w.models))
    assert min(st.error_bounds()) > TOL
    ids = ids_dev(torch, w.image_ids)
    d = st.decode_batch_ex(ids, 40, 40)
    for flag in (rinr.FLAG_FP16_ACT, rinr.FLAG_FP16_ALL):
        assert torch.equal(st.decode_batch_ex(ids, 40, 40, rinr.OUT_F32, flag), d)
        assert st.last_launch_info()["kernels"] == rinr.FAMILIES[0]
        forced = st.decode_batch_ex(ids, 40, 40, rinr.OUT_F32, flag | UNCHECKED)
        assert not torch.equal(forced, d)
    st.close()


@pytest.mark.parametrize("w0,lo,hi", [(30.0, -0.25, 1.5), (10.0, -1.0, 1.0), (55.5, 0.0, 1.0), (17.25, -2.0, 0.5), (30.0, 1.0, -1.0)])
def test_other_frequencies_and_coordinate_ranges(torch, w0, lo, hi):
    """The sine frequency (Sec. V-B sweeps it) and the coordinate range are store options: frequencies other than 30,
    ranges that are not symmetric, not of unit length, and reversed."""
    ms = synth.make_models(41, np.arange(5), 32, 4, [0, 8, 6, 8, 0], 0.6, w0=w0) + synth.make_models(42, np.arange(3), 64, 3, [0, 0, 16, 0], 0.8, w0=w0)
    w = synth.Workload("w0/range", ms, np.array([7, 1, 4, 0, 6, 2]), 29, 43, False, w0, lo, hi)
    check_workload(torch, w)
    check_workload(torch, w, models=image_like(ms), u8=True)


def test_decode_argument_errors(torch):
    w = synth.workload(2, n_images=2)
    st = rinr.Store(rinr.pack(w.models))
    L = rinr.lib()
    ids = ids_dev(torch, w.image_ids)
    out = torch.empty((2, 3, 4, 4), device="cuda")
    h = st._h
    assert L.rinr_decode_batch(None, ids.data_ptr(), 2, 4, 4, out.data_ptr(), None) == rinr.E_NULL
    assert L.rinr_decode_batch(h, None, 2, 4, 4, out.data_ptr(), None) == rinr.E_NULL
    assert L.rinr_decode_batch(h, ids.data_ptr(), 2, 4, 4, None, None) == rinr.E_NULL
    assert L.rinr_decode_batch(h, ids.data_ptr(), -1, 4, 4, out.data_ptr(), None) == rinr.E_ARG
    assert L.rinr_decode_batch(h, ids.data_ptr(), 2, 0, 4, out.data_ptr(), None) == rinr.E_ARG
    assert L.rinr_decode_batch(h, ids.data_ptr(), 2, 4, -3, out.data_ptr(), None) == rinr.E_ARG
    assert L.rinr_decode_batch(h, ids.data_ptr(), 2, 1 << 16, 1 << 16, out.data_ptr(), None) == rinr.E_SIZE
    assert L.rinr_decode_batch(h, ids.data_ptr(), 2, 4, 4, out.data_ptr() + 2, None) == rinr.E_ALIGN
    o = rinr.DecodeOpts(7, 0, None)
    assert L.rinr_decode_batch_ex(h, ids.data_ptr(), 2, 4, 4, out.data_ptr(), C.byref(o), None) == rinr.E_ARG
    o = rinr.DecodeOpts(rinr.OUT_U8, rinr.FLAG_NO_CLAMP, None)
    assert L.rinr_decode_batch_ex(h, ids.data_ptr(), 2, 4, 4, out.data_ptr(), C.byref(o), None) == rinr.E_ARG
    o = rinr.DecodeOpts(rinr.OUT_F32_AND_U8, 0, None)
    assert L.rinr_decode_batch_ex(h, ids.data_ptr(), 2, 4, 4, out.data_ptr(), C.byref(o), None) == rinr.E_NULL
    assert L.rinr_decode_batch_ex(h, ids.data_ptr(), 2, 4, 4, out.data_ptr(), None, None) == rinr.E_NULL
    assert L.rinr_debug_dequant(h, 5, 0, out.data_ptr(), None, None) == rinr.E_ARG
    assert L.rinr_debug_dequant(h, 0, 9, out.data_ptr(), None, None) == rinr.E_ARG
    assert L.rinr_store_open(st.dev_blob.data_ptr() + 4, None, 64, C.byref(C.c_void_p())) == rinr.E_ALIGN
    st.close()


def test_heaviest_first_order_changes_nothing(torch):
    """With a workspace the slots of a ragged batch are taken heaviest model first: same bytes out, in every mode,
    with repeats and out-of-range ids in the batch; a store of one width ignores the workspace."""
    w = synth.workload(5, n_images=300, pool=500, H=24, W=37)
    st = rinr.Store(rinr.pack(w.models, w.w0, w.coord_lo, w.coord_hi))
    ids_h = w.image_ids.copy()
    ids_h[[3, 77, 299]] = [-1, 500, 2 ** 40]
    ids = torch.from_numpy(ids_h).cuda()
    ws = torch.empty(rinr.workspace_bytes(300), dtype=torch.uint8, device="cuda")
    for mode in (0, rinr.FLAG_FP32_MFMA, rinr.FLAG_FP16_ACT, rinr.FLAG_FP16_ALL):
        a = st.decode_batch_ex(ids, 24, 37, rinr.OUT_F32, mode)
        b = st.decode_batch_ex(ids, 24, 37, rinr.OUT_F32, mode, workspace=ws)
        assert torch.equal(a, b), mode
        order = ws[:1200].view(torch.int32).cpu().numpy()
        assert np.array_equal(np.sort(order), np.arange(300))              # a permutation of the slots ...
        cost = np.array([0 if not (0 <= i < 500) else (len(w.models[int(i)].layers)) *
                         {1: 3, 2: 6, 3: 10, 4: 13}[(max(ly.n_out for ly in w.models[int(i)].layers[:-1]) + 15) // 16] for i in ids_h])
        assert np.all(np.diff(cost[order]) <= 0)                            # ... by falling cost
        f32, u8 = st.decode_batch_ex(ids, 24, 37, rinr.OUT_F32_AND_U8, mode & rinr.FLAG_FP32_MFMA, workspace=ws)
        assert torch.equal(f32, st.decode_batch_ex(ids, 24, 37, rinr.OUT_F32, mode & rinr.FLAG_FP32_MFMA))
    assert st.status() == 3 * 4 * 4                 # three bad ids in each of the four decodes per mode
    # too small a workspace, a misaligned one
    L = rinr.lib()
    out = torch.empty((300, 3, 24, 37), device="cuda")
    o = rinr.DecodeOpts(rinr.OUT_F32, 0, None)
    o.workspace, o.workspace_bytes = ws.data_ptr(), 300 * 4 - 1
    assert L.rinr_decode_batch_ex(st._h, ids.data_ptr(), 300, 24, 37, out.data_ptr(), C.byref(o), None) == rinr.E_SIZE
    o.workspace, o.workspace_bytes = ws.data_ptr() + 2, 300 * 4
    assert L.rinr_decode_batch_ex(st._h, ids.data_ptr(), 300, 24, 37, out.data_ptr(), C.byref(o), None) == rinr.E_ALIGN
    st.close()
    # one width, several depths: ordered too
    rng = np.random.default_rng(5)
    deep = []
    for k in range(40):
        dims = [2] + [32] * int(rng.integers(1, 6)) + [3]
        deep.append(Model([Layer(dims[l], dims[l + 1], 0, 0.0, 0, (rng.uniform(-1, 1, (dims[l + 1], dims[l])) * (0.5 if l == 0 else 0.03)).astype(np.float32),
                                 None, rng.uniform(-.1, .1, dims[l + 1]).astype(np.float32)) for l in range(len(dims) - 1)]))
    st3 = rinr.Store(rinr.pack(deep))
    ids3 = torch.from_numpy(rng.integers(0, 40, 100)).cuda()
    plain = st3.decode_batch_ex(ids3, 20, 20)
    assert st3.last_launch_info()["launches"] == 1
    assert torch.equal(st3.decode_batch_ex(ids3, 20, 20, workspace=ws), plain)
    assert st3.last_launch_info()["launches"] == 2
    depth = np.array([len(deep[int(i)].layers) for i in ids3.cpu().numpy()])
    assert np.all(np.diff(depth[ws[:400].view(torch.int32).cpu().numpy()]) <= 0)
    st3.close()
    w2 = synth.workload(2, n_images=20, H=16, W=16)
    st2 = rinr.Store(rinr.pack(w2.models))
    ids2 = torch.from_numpy(w2.image_ids).cuda()
    ws.fill_(255)
    assert torch.equal(st2.decode_batch_ex(ids2, 16, 16, workspace=ws), st2.decode_batch_ex(ids2, 16, 16))
    assert int(ws.min()) == 255                                              # untouched
    st2.close()


def test_zz_report_worst_errors():
    names = {0: "default", rinr.FLAG_FP32_MFMA: "fp32 MFMA", rinr.FLAG_FP16_ACT: "fp16 activations where granted",
             rinr.FLAG_FP16_ALL: "fp16 weights and activations where granted", rinr.FLAG_FP16_ACT | UNCHECKED: "fp16 activations forced",
             rinr.FLAG_FP16_ALL | UNCHECKED: "fp16 weights and activations forced"}
    print("largest unclamped max-abs error per mode:", {names[m]: f"{e:.2e}" for m, e in WORST.items()})
