"""The hardware probes read what they say they read: the tile-load probe's checksum is recomputed on the host
(tile order, wrap-around of the tile index, both load paths), the copy probe copies, bad sizes are refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1811_05233_amd as P                     # noqa: E402
from paper_1811_05233_amd import synth               # noqa: E402
from gpu_util import DEV, host                       # noqa: E402

TILE_HALFS = 8192


def expected(src, ntiles, blocks, iters, stride, through_lds):
    """Block b walks iters tiles from tile (b*stride) % ntiles.  LDS path: out[b*256+t] = sum of half t*8 of every tile.
    Vector path: XOR of the 32-bit words t*4..t*4+3 of each 4 KB quarter of every tile."""
    halves = src.reshape(ntiles, TILE_HALFS).astype(np.float32)
    words = src.view(np.uint32).reshape(ntiles, 4, 256, 4)
    t = np.arange(256)
    out = []
    for b in range(blocks):
        tile = (b * stride) % ntiles
        acc = np.zeros(256, np.float32) if through_lds else np.zeros(256, np.uint32)
        for _ in range(iters):
            if through_lds:
                acc = acc + halves[tile, t * 8]
            else:
                acc = acc ^ np.bitwise_xor.reduce(np.bitwise_xor.reduce(words[tile], axis=2), axis=0)
            tile = (tile + 1) % ntiles
        out.append(acc)
    return np.concatenate(out)


@pytest.mark.parametrize("ntiles,blocks,iters,stride", [(3, 5, 7, 7), (1, 2, 1, 0), (16, 9, 2, 5), (4, 3, 40, 1), (8, 4, 2, 2)])
def test_tile_load_probe_checksums(ntiles, blocks, iters, stride):
    print("[case] tile probe ntiles=%d blocks=%d iters=%d stride=%d" % (ntiles, blocks, iters, stride), flush=True)
    # small integers: every partial sum is exact in FP32, so the order of additions does not matter
    src = (synth.labels(700 + ntiles, ntiles * TILE_HALFS, 17).astype(np.float32) - 8.0).astype(np.float16)
    d_src = torch.from_numpy(src).to(DEV)
    for through_lds in (1, 0):
        out = torch.full((blocks * 256,), float("nan"), dtype=torch.float32, device=DEV)
        P.probe_tile_load(d_src, src.nbytes, blocks, iters, stride, through_lds, out)
        torch.cuda.synchronize()
        want = expected(src, ntiles, blocks, iters, stride, through_lds)
        if through_lds:
            assert np.array_equal(out.cpu().numpy(), want)
        else:
            assert np.array_equal(out.view(torch.int32).cpu().numpy().view(np.uint32), want)


def test_mfma_copy_and_empty_probes():
    out = torch.full((4 * 256,), float("nan"), dtype=torch.float32, device=DEV)
    P.probe_mfma(4, 3, out)
    torch.cuda.synchronize()
    assert np.all(np.isfinite(host(out)))
    src = torch.from_numpy(synth.normal_f32(710, (4096 + 4,))).to(DEV)
    dst = torch.zeros_like(src)
    P.probe_copy(src, dst, src.numel() * 4)
    P.probe_empty(3)
    torch.cuda.synchronize()
    assert np.array_equal(host(dst), host(src))


def test_probe_sizes_are_checked():
    buf = torch.zeros(TILE_HALFS, dtype=torch.float16, device=DEV)
    out = torch.zeros(256, dtype=torch.float32, device=DEV)
    with pytest.raises(P.Rn50Error):
        P.probe_tile_load(buf, 16384 - 16, 1, 1, 1, 1, out)       # not a whole tile
    with pytest.raises(P.Rn50Error):
        P.probe_tile_load(buf, 16384, 0, 1, 1, 1, out)
    with pytest.raises(P.Rn50Error):
        P.probe_mfma(1, 0, out)
    with pytest.raises(P.Rn50Error):
        P.probe_copy(buf, buf, 24)
    with pytest.raises(P.Rn50Error):
        P.probe_empty(0)
