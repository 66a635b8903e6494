"""GPU check of bn_relu_fwd_static, the entry point for callers that cannot allocate: it runs the kernels of
bn_relu_fwd on a device array inside the library instead of a workspace argument, so its results must equal
bn_relu_fwd's bit for bit.  Two calls in a row, the second on a smaller input (the array keeps the first call's
contents), then the size limit."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1811_05233_amd as P                     # noqa: E402
from paper_1811_05233_amd import synth               # noqa: E402
from gpu_util import DEV, dev_f, dev_h, host         # noqa: E402


def both(m, c, relu, res, seed):
    print("[case] bn_relu_fwd_static m=%d c=%d relu=%d res=%d" % (m, c, relu, res), flush=True)
    x = dev_h(synth.normal_f16(seed, (m, c)) * 1.5 + 0.25)
    r = dev_h(synth.normal_f16(seed + 1, (m, c))) if res else None
    g = dev_f(1.0 + 0.1 * synth.normal_f32(seed + 2, (c,)))
    b = dev_f(0.1 * synth.normal_f32(seed + 3, (c,)))
    d = P.make_bn_desc(m, c, 1e-5, relu, res)
    outs = []
    for fn in (P.bn_relu_fwd, P.bn_relu_fwd_static):
        y = torch.full((m, c), float("nan"), dtype=torch.float16, device=DEV)
        mean = torch.full((c,), float("nan"), dtype=torch.float32, device=DEV)
        inv = torch.full((c,), float("nan"), dtype=torch.float32, device=DEV)
        fn(d, x, g, b, r, y, mean, inv)
        outs.append((host(y), host(mean), host(inv)))
    for a, e in zip(outs[1], outs[0]):
        assert np.all(np.isfinite(e)) and np.array_equal(a, e)


def test_static_entry_point_matches_workspace_entry_point_twice():
    both(50000, 256, True, True, 900)        # 2048 partial rows: the whole array is written
    both(777, 64, True, False, 910)          # smaller input on the array the first call left behind
    both(9, 8, False, False, 920)


def test_static_entry_point_rejects_what_does_not_fit():
    l = P.lib()
    t = torch.zeros(1 << 12, dtype=torch.float16, device=DEV)
    f = torch.zeros(1 << 12, dtype=torch.float32, device=DEV)
    d = P.make_bn_desc(2, 512)
    rc = l.bn_relu_fwd_static(ctypes.byref(d), t.data_ptr(), f.data_ptr(), f.data_ptr(), None, t.data_ptr(),
                              f.data_ptr(), f.data_ptr(), None)
    assert rc == -4                          # RN50_ERR_WORKSPACE: beyond RN50_BN_STATIC_MAX_C channels
    d = P.make_bn_desc(2, 24)
    assert l.bn_relu_fwd_static(ctypes.byref(d), t.data_ptr(), f.data_ptr(), f.data_ptr(), None, t.data_ptr(),
                                f.data_ptr(), f.data_ptr(), None) == -2
