"""GPU parity: conv_fwd / conv_dgrad / conv_wgrad against the CPU oracle (FP64 instantiation)
on identical FP16-representable inputs.  Tolerance 2e-2 relative to max(|ref|, 1e-2*max|ref|)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import oracle as O                                   # noqa: E402
import paper_1811_05233_amd as P                     # noqa: E402
from paper_1811_05233_amd import synth               # noqa: E402
from gpu_util import DEV, dev_h, host, rel_err       # noqa: E402

TOL16 = 2e-2

# The 23 distinct convolution shapes of ResNet-50 v1.5: (cin, cout, r, stride, pad, hin)
RESNET50_SHAPES = [
    (3, 64, 7, 2, 3, 224), (64, 64, 1, 1, 0, 56), (64, 64, 3, 1, 1, 56), (64, 256, 1, 1, 0, 56),
    (256, 64, 1, 1, 0, 56), (256, 128, 1, 1, 0, 56), (128, 128, 3, 2, 1, 56), (128, 512, 1, 1, 0, 28),
    (256, 512, 1, 2, 0, 56), (512, 128, 1, 1, 0, 28), (128, 128, 3, 1, 1, 28), (512, 256, 1, 1, 0, 28),
    (256, 256, 3, 2, 1, 28), (256, 1024, 1, 1, 0, 14), (512, 1024, 1, 2, 0, 28), (1024, 256, 1, 1, 0, 14),
    (256, 256, 3, 1, 1, 14), (1024, 512, 1, 1, 0, 14), (512, 512, 3, 2, 1, 14), (512, 2048, 1, 1, 0, 7),
    (1024, 2048, 1, 2, 0, 14), (2048, 512, 1, 1, 0, 7), (512, 512, 3, 1, 1, 7)]

# ragged / degenerate geometry: (n, h, w, cin, cout, r, stride, pad)
EDGE_SHAPES = [
    (1, 1, 1, 64, 64, 1, 1, 0), (1, 1, 1, 64, 64, 3, 1, 1), (3, 7, 9, 64, 128, 3, 2, 1), (2, 9, 7, 128, 64, 3, 1, 1),
    (1, 5, 5, 64, 64, 1, 2, 0), (5, 13, 11, 64, 192, 3, 1, 1), (2, 10, 6, 3, 64, 7, 2, 3), (1, 2, 2, 3, 128, 7, 2, 3),
    (1, 33, 31, 192, 64, 3, 2, 1), (2, 3, 3, 64, 64, 3, 2, 1)]


def run_case(n, h, w, cin, cout, r, stride, pad, seed, do_dgrad=True):
    print("[case] conv n=%d h=%d w=%d c=%d k=%d r=%d stride=%d pad=%d" % (n, h, w, cin, cout, r, stride, pad), flush=True)
    x = synth.normal_f16(seed, (n, h, w, cin))
    wt = synth.he_normal_f16(seed + 1, (cout, r, r, cin), cin * r * r)
    p, q = O.out_hw(h, w, r, r, stride, pad)
    dy = synth.normal_f16(seed + 2, (n, p, q, cout))
    d = P.make_conv_desc(n, h, w, cin, cout, r, r, stride, pad)
    xd, wd, dyd = dev_h(x), dev_h(wt), dev_h(dy)
    f64 = np.float64

    y = torch.full((n, p, q, cout), float("nan"), dtype=torch.float16, device=DEV)
    P.conv_fwd(d, xd, wd, y)
    ry = O.conv_fwd(x.astype(f64), wt.astype(f64), stride, pad)
    e = rel_err(host(y), ry)
    assert e <= TOL16, "fwd err %g" % e

    dw = torch.full((cout, r, r, cin), float("nan"), dtype=torch.float16, device=DEV)
    P.conv_wgrad(d, xd, dyd, dw)
    rdw = O.conv_wgrad(x.astype(f64), dy.astype(f64), wt.shape, stride, pad)
    e = rel_err(host(dw), rdw)
    assert e <= TOL16, "wgrad err %g" % e

    if do_dgrad:
        dx = torch.full((n, h, w, cin), float("nan"), dtype=torch.float16, device=DEV)
        P.conv_dgrad(d, dyd, wd, dx)
        rdx = O.conv_dgrad(dy.astype(f64), wt.astype(f64), x.shape, stride, pad)
        e = rel_err(host(dx), rdx)
        assert e <= TOL16, "dgrad err %g" % e
        # positions no filter tap reaches are exactly zero
        assert np.array_equal(host(dx) == 0, rdx == 0) or np.all(host(dx)[rdx == 0] == 0)


@pytest.mark.parametrize("shape", RESNET50_SHAPES)
def test_conv_resnet50_shapes_batch2(shape):
    cin, cout, r, stride, pad, hin = shape
    run_case(2, hin, hin, cin, cout, r, stride, pad, 100 + RESNET50_SHAPES.index(shape) * 3, do_dgrad=cin != 3)


@pytest.mark.parametrize("shape", EDGE_SHAPES)
def test_conv_edge_shapes(shape):
    n, h, w, cin, cout, r, stride, pad = shape
    run_case(n, h, w, cin, cout, r, stride, pad, 300 + EDGE_SHAPES.index(shape) * 3, do_dgrad=cin != 3)


# every kernel variant, named through the *_variant entry points, on shapes where each applies: (n, h, w, cin, cout, r, stride, pad).
# Small images make one tile span several of them, and most shapes end in a ragged tile.
VARIANT_SHAPES = [
    (3, 14, 14, 128, 128, 3, 1, 1), (5, 7, 7, 64, 256, 3, 1, 1), (2, 28, 28, 96 + 32, 64, 3, 1, 1),
    (2, 56, 56, 64, 64, 3, 1, 1), (7, 5, 3, 64, 128, 3, 1, 1), (1, 6, 70, 64, 64, 3, 1, 1), (40, 2, 2, 64, 64, 3, 1, 1),
    (2, 14, 14, 256, 256, 1, 1, 0), (2, 15, 13, 128, 128, 3, 2, 1)]
MAX_GATHER_TILES, MAX_WGRAD_VARIANTS = 24, 60     # parametrisation bounds; the library reports the real counts


@pytest.mark.parametrize("tile", range(MAX_GATHER_TILES))
def test_conv_every_gather_tile(tile):
    if tile >= P.conv_variant_count(P.CONV_FWD):
        pytest.skip("the library has fewer gather-GEMM tiles")
    for i, (n, h, w, cin, cout, r, stride, pad) in enumerate(VARIANT_SHAPES):
        print("[case] tile=%d n=%d h=%d w=%d c=%d k=%d r=%d stride=%d" % (tile, n, h, w, cin, cout, r, stride), flush=True)
        x = synth.normal_f16(700 + i, (n, h, w, cin))
        wt = synth.he_normal_f16(720 + i, (cout, r, r, cin), cin * r * r)
        p, q = O.out_hw(h, w, r, r, stride, pad)
        dy = synth.normal_f16(740 + i, (n, p, q, cout))
        d = P.make_conv_desc(n, h, w, cin, cout, r, r, stride, pad)
        y = torch.full((n, p, q, cout), float("nan"), dtype=torch.float16, device=DEV)
        P.conv_fwd(d, dev_h(x), dev_h(wt), y, variant=tile)
        e = rel_err(host(y), O.conv_fwd(x.astype(np.float64), wt.astype(np.float64), stride, pad))
        assert e <= TOL16, "fwd err %g (tile %d, shape %d)" % (e, tile, i)
        dx = torch.full((n, h, w, cin), float("nan"), dtype=torch.float16, device=DEV)
        P.conv_dgrad(d, dev_h(dy), dev_h(wt), dx, variant=tile)
        e = rel_err(host(dx), O.conv_dgrad(dy.astype(np.float64), wt.astype(np.float64), x.shape, stride, pad))
        assert e <= TOL16, "dgrad err %g (tile %d, shape %d)" % (e, tile, i)


def test_stem_forward_through_every_tile_that_fits_it():
    """The 7x7 / stride 2 stem goes through the 32-wide tiles with 64 columns; every id runs (the others fall back)."""
    shapes = [(3, 34, 30, 3, 64, 7, 2, 3), (2, 64, 64, 3, 64, 7, 2, 3)]
    applies = [v for v in range(P.conv_variant_count(P.CONV_FWD))
               if P.conv_variant_applies(P.make_conv_desc(*shapes[0][:5], 7, 7, 2, 3), P.CONV_FWD, v)]
    assert len(applies) == 4
    for i, (n, h, w, cin, cout, r, stride, pad) in enumerate(shapes):
        x = synth.normal_f16(780 + i, (n, h, w, cin))
        wt = synth.he_normal_f16(790 + i, (cout, r, r, cin), cin * r * r)
        ref = O.conv_fwd(x.astype(np.float64), wt.astype(np.float64), stride, pad)
        p, q = O.out_hw(h, w, r, r, stride, pad)
        d = P.make_conv_desc(n, h, w, cin, cout, r, r, stride, pad)
        for v in applies + [applies[0] + 1]:
            print("[case] stem tile=%d shape %d" % (v, i), flush=True)
            y = torch.full((n, p, q, cout), float("nan"), dtype=torch.float16, device=DEV)
            P.conv_fwd(d, dev_h(x), dev_h(wt), y, variant=v)
            e = rel_err(host(y), ref)
            assert e <= TOL16, "stem fwd err %g (tile %d, shape %d)" % (e, v, i)


@pytest.mark.parametrize("variant", range(MAX_WGRAD_VARIANTS))
def test_conv_every_wgrad_variant(variant):
    if variant >= P.conv_variant_count(P.CONV_WGRAD):
        pytest.skip("the library has fewer filter-gradient variants")
    for i, (n, h, w, cin, cout, r, stride, pad) in enumerate(VARIANT_SHAPES):
        print("[case] wgrad variant=%d shape %d" % (variant, i), flush=True)
        x = synth.normal_f16(760 + i, (n, h, w, cin))
        p, q = O.out_hw(h, w, r, r, stride, pad)
        dy = synth.normal_f16(780 + i, (n, p, q, cout))
        d = P.make_conv_desc(n, h, w, cin, cout, r, r, stride, pad)
        dw = torch.full((cout, r, r, cin), float("nan"), dtype=torch.float16, device=DEV)
        P.conv_wgrad(d, dev_h(x), dev_h(dy), dw, variant=variant)
        e = rel_err(host(dw), O.conv_wgrad(x.astype(np.float64), dy.astype(np.float64), (cout, r, r, cin), stride, pad))
        assert e <= TOL16, "wgrad err %g (variant %d, shape %d)" % (e, variant, i)


def test_conv_fwd_deterministic_and_delta_filter():
    n, h, w, c = 2, 12, 10, 64
    x = synth.normal_f16(380, (n, h, w, c))
    f = np.zeros((c, 3, 3, c), np.float32)
    for i in range(c):
        f[i, 1, 1, i] = 1.0
    d = P.make_conv_desc(n, h, w, c, c, 3, 3, 1, 1)
    xd, fd = dev_h(x), dev_h(f)
    y1 = torch.zeros(n, h, w, c, dtype=torch.float16, device=DEV)
    y2 = torch.zeros_like(y1)
    P.conv_fwd(d, xd, fd, y1)
    P.conv_fwd(d, xd, fd, y2)
    assert np.array_equal(host(y1), x.astype(np.float64)) and np.array_equal(host(y1), host(y2))


def test_conv_error_paths():
    t = torch.zeros(1 << 16, dtype=torch.float16, device=DEV)
    ws = torch.zeros(1 << 22, dtype=torch.uint8, device=DEV)
    for bad in [P.make_conv_desc(1, 8, 8, 60, 64, 1, 1, 1, 0), P.make_conv_desc(1, 8, 8, 64, 64, 5, 5, 1, 2),
                P.make_conv_desc(1, 8, 8, 64, 64, 3, 3, 3, 1), P.make_conv_desc(0, 8, 8, 64, 64, 1, 1, 1, 0),
                P.make_conv_desc(1, 8, 8, 64, 64, 1, 1, 1, 0, dt=P.RN50_BF16)]:
        with pytest.raises(P.Rn50Error):
            P.conv_fwd(bad, t, t, t, ws)
    stem = P.make_conv_desc(1, 8, 8, 3, 64, 7, 7, 2, 3)
    with pytest.raises(P.Rn50Error):
        P.conv_dgrad(stem, t, t, t, ws)
    with pytest.raises(P.Rn50Error):                 # workspace too small for the transposed filter
        P.conv_dgrad(P.make_conv_desc(1, 8, 8, 64, 64, 3, 3, 1, 1), t, t, t, torch.zeros(16, dtype=torch.uint8, device=DEV))
