"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, validates arguments before touching the GPU, and its flat parameter layout agrees
with the oracle's independently written one."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1811_05233_amd as P
from oracle import resnet50 as R

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "rn50.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b([a-z][a-z0-9_]*)\s*\(", src)
    return sorted(set(n for n in names if n not in ("defined",)))


def test_library_exports_every_declared_symbol():
    l = ctypes.CDLL(P.LIB_PATH)
    declared = header_functions()
    assert "rn50_step" in declared and "conv_wgrad" in declared and len(declared) >= 20
    for name in declared:
        assert hasattr(l, name), name
    assert set(P.EXPORTS) == set(declared)
    P.lib()


def test_status_strings():
    l = P.lib()
    assert l.rn50_status_string(0) == b"ok"
    for rc in range(-6, 0):
        assert len(l.rn50_status_string(rc)) > 0


@pytest.mark.parametrize("kw", [
    dict(batch=32), dict(batch=2, image_hw=(56, 56), has_stem=False, blocks=(1,)),
    dict(batch=4, image_hw=(64, 64), blocks=(1, 1, 1, 1)), dict(batch=1, image_hw=(32, 32), blocks=(2, 1), base_width=128, classes=16)])
def test_flat_layout_matches_oracle(kw):
    cfg = P.make_config(**kw)
    net = R.Net(kw["batch"], kw.get("image_hw", (224, 224)), kw.get("has_stem", True), kw.get("blocks", (3, 4, 6, 3)),
                kw.get("base_width", 64), kw.get("classes", 1000))
    lay = P.rn50_param_layout(cfg)
    assert P.rn50_param_count(cfg) == net.param_count
    assert lay == [(s.kind, s.offset, s.count, s.fan_in) for s in net.segments]
    assert P.rn50_workspace_bytes(cfg) > 0


def test_resnet50_param_count():
    assert P.rn50_param_count(P.make_config(32)) == 25557032


def test_bad_configs_and_null_arguments():
    l = P.lib()
    for kw in [dict(batch=0), dict(batch=2, base_width=48), dict(batch=2, classes=1001), dict(batch=2, image_hw=(223, 224)),
               dict(batch=2, blocks=(0,)), dict(batch=2, dt=P.RN50_BF16)]:
        cfg = P.make_config(**kw)
        assert P.rn50_param_count(cfg) == 0 and P.rn50_workspace_bytes(cfg) == 0
        h = ctypes.c_void_p()
        assert l.rn50_create(ctypes.byref(h), ctypes.byref(cfg), None, 0) < 0
    cfg = P.make_config(2, (56, 56), False, (1,))
    h = ctypes.c_void_p()
    assert l.rn50_create(ctypes.byref(h), ctypes.byref(cfg), None, 0) == -4          # workspace
    assert l.rn50_create(None, ctypes.byref(cfg), None, 0) == -1
    assert l.rn50_step(None, None, None, None, None, None, None, None, None, None) == -1
    # kernels: validation happens before any launch, so these run without a GPU
    d = P.make_conv_desc(1, 8, 8, 60, 64, 1, 1, 1, 0)
    assert l.conv_fwd(ctypes.byref(d), None, None, None, None, 0, None) == -2
    d = P.make_conv_desc(1, 8, 8, 64, 64, 1, 1, 1, 0)
    assert l.conv_fwd(ctypes.byref(d), None, None, None, None, 0, None) == -1
    assert l.conv_fwd(ctypes.byref(d), 16, 32, 8, None, 0, None) == -5              # misaligned y
    assert P.conv_workspace_bytes(d, P.CONV_DGRAD) == 64 * 64 * 2
    assert l.conv_dgrad(ctypes.byref(d), 16, 32, 48, None, 0, None) == -4
    b = P.make_bn_desc(10, 12)
    assert l.bn_relu_fwd(ctypes.byref(b), None, None, None, None, None, None, None, None, 0, None) == -2
    assert l.ls_xent_fwd_bwd(0, 10, None, None, 0.1, 1.0, None, None, None, 0, None) == -2
    assert l.ls_xent_fwd_bwd(4, 10, None, None, 0.1, 1.0, None, None, None, 1, None) == -3
    assert l.sgd_momentum_flat(8, None, 0, 1.0, None, None, None, 0.1, 0.9, 0.0, None) == -1
    assert l.sgd_momentum_flat(0, None, 0, 1.0, None, None, None, 0.1, 0.9, 0.0, None) == 0


def test_bn_channel_counts_the_header_states():
    """bn_*: c a power of two from 8 to 2048 or a multiple of 2048; the static-scratch form up to 256 channels."""
    l = P.lib()
    for c, ok in [(8, True), (64, True), (2048, True), (4096, True), (6144, True), (24, False), (192, False), (320, False),
                  (3072, False), (4, False), (0, False)]:
        b = P.make_bn_desc(10, c)
        assert (P.bn_workspace_bytes(b) > 0) == ok, c
        rc = l.bn_relu_fwd(ctypes.byref(b), None, None, None, None, None, None, None, None, 0, None)
        assert rc == (-1 if ok else -2), (c, rc)                     # shape is judged before the pointers
    b = P.make_bn_desc(10, 512)
    assert l.bn_relu_fwd_static(ctypes.byref(b), None, None, None, None, None, None, None, None) == -4
    b = P.make_bn_desc(10, 256)
    assert l.bn_relu_fwd_static(ctypes.byref(b), None, None, None, None, None, None, None, None) == -1
    assert P.conv_variant_count(P.CONV_FWD) >= 12 and P.conv_variant_count(P.CONV_WGRAD) >= 30 and P.conv_variant_count(7) == 0


def test_lars_table_validation_without_a_gpu():
    """lars_workspace_bytes / lars_plan_create reject bad segment tables before anything touches the device."""
    l = P.lib()

    def table(segs):
        return (P.rn50_lars_segment * len(segs))(*[P.rn50_lars_segment(o, c, u) for o, c, u in segs]), len(segs)

    good, n = table([(0, 1000, 1), (1000, 24, 0), (1024, 5000, 1)])
    need = l.lars_workspace_bytes(good, n)
    assert need > 0 and need % 256 == 0
    assert l.lars_workspace_bytes(None, 0) > 0                       # an empty table is a valid (no-op) plan
    bad_align, nb = table([(4, 8, 1)])
    assert l.lars_workspace_bytes(bad_align, nb) == 0
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(1 << 20)                                  # aligned, never dereferenced on these paths
    assert l.lars_plan_create(ctypes.byref(h), bad_align, nb, fake, 1 << 20) == -2 and not h.value      # RN50_ERR_SHAPE
    overlap, no = table([(0, 16, 1), (8, 16, 0)])
    assert l.lars_plan_create(ctypes.byref(h), overlap, no, fake, 1 << 20) == -2 and not h.value
    assert l.lars_plan_create(ctypes.byref(h), good, n, None, 0) == -4                                  # RN50_ERR_WORKSPACE
    assert l.lars_plan_create(ctypes.byref(h), good, n, fake, need - 1) == -4
    assert l.lars_plan_create(ctypes.byref(h), good, n, ctypes.c_void_p((1 << 20) + 4), need) == -5     # RN50_ERR_ALIGN
    assert l.lars_plan_create(None, good, n, fake, need) == -1                                          # RN50_ERR_NULL
    assert l.lars_momentum_flat(None, fake, 0, 1.0, fake, fake, None, 0.1, 0.9, 0.0, 0.01, 1e-6, None, None) == -1
    l.lars_plan_destroy(None)


def test_schedule_functions_match_the_oracle():
    from oracle import schedule as S
    for e in np.linspace(0, 90, 361):
        assert abs(P.sched_lr_b(e) - S.lr_b(e)) <= 1e-12 * max(1.0, S.lr_b(e))
        if e < 90:
            for b in (32768, 55296, 65536, 121856):
                assert abs(P.sched_momentum_b(e, b) - S.momentum_b(e, b)) <= 1e-12
        for x in range(5):
            assert P.sched_batch(x, e) == S.batch(x, e)
    assert abs(P.sched_momentum_b(90, 55296) - 0.83125) < 1e-12       # LR = 0: the constant ratio is used
    for bad in [(5, 1.0), (-1, 1.0), (2, -0.5), (2, 90.5), (2, float("nan"))]:
        with pytest.raises(P.Rn50Error):
            P.sched_batch(*bad)


def test_which_variants_apply_to_which_shapes():
    """rn50_conv_variant_applies launches nothing: the strip kernels are for 3x3 / stride 1 / pad 1 up to 56 columns,
    128-column tiles need the output width of the GEMM to be a multiple of 128, wide K-slabs a matching reduction
    length; out-of-range ids and the stem's data gradient never apply."""
    nf = P.conv_variant_count(P.CONV_FWD)
    nw = P.conv_variant_count(P.CONV_WGRAD)
    c33 = P.make_conv_desc(4, 56, 56, 64, 64, 3, 3, 1, 1)
    c33s2 = P.make_conv_desc(4, 56, 56, 128, 128, 3, 3, 2, 1)
    c11 = P.make_conv_desc(4, 14, 14, 1024, 256, 1, 1, 1, 0)
    stem = P.make_conv_desc(4, 224, 224, 3, 64, 7, 7, 2, 3)
    strips = [v for v in range(nf) if P.conv_variant_applies(c33, P.CONV_FWD, v) and not P.conv_variant_applies(c33s2, P.CONV_FWD, v)
              and not P.conv_variant_applies(c11, P.CONV_FWD, v)]
    assert len(strips) == 6                                  # three tile heights x (ring, single stage)
    for v in strips:
        assert P.conv_variant_applies(c33, P.CONV_DGRAD, v) and not P.conv_variant_applies(c33s2, P.CONV_DGRAD, v)
    # 64 output channels: no 128-column tile; 256 output channels (forward) / 1024 (data gradient): all of them
    n64 = sum(P.conv_variant_applies(c33, P.CONV_FWD, v) for v in range(nf))
    n256 = sum(P.conv_variant_applies(c11, P.CONV_FWD, v) for v in range(nf))
    assert 0 < n64 - 6 < n256 == nf - 6
    assert sum(P.conv_variant_applies(stem, P.CONV_FWD, v) for v in range(nf)) == 4      # the 32-wide, 64-column tiles
    assert not any(P.conv_variant_applies(stem, P.CONV_DGRAD, v) for v in range(nf))
    for d in (c33, c11):
        assert not P.conv_variant_applies(d, P.CONV_FWD, -1) and not P.conv_variant_applies(d, P.CONV_FWD, nf)
        assert not P.conv_variant_applies(d, P.CONV_WGRAD, nw)
    wstrips = [v for v in range(nw) if P.conv_variant_applies(c33, P.CONV_WGRAD, v) and not P.conv_variant_applies(c11, P.CONV_WGRAD, v)]
    assert len(wstrips) >= 3 and all(not P.conv_variant_applies(c33s2, P.CONV_WGRAD, v) for v in wstrips[-3:])
