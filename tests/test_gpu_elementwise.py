"""GPU parity: sgd_momentum_flat, ls_xent_fwd_bwd, bn_relu_fwd/bwd against the CPU oracle.

Tolerances: 1e-5 relative for the FP32 loss and update, 2e-2 (relative to
max(|ref|, 1e-2*max|ref|)) for FP16 tensors; saved BN statistics 1e-4."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import oracle as O                                   # noqa: E402
import paper_1811_05233_amd as P                     # noqa: E402
from paper_1811_05233_amd import synth               # noqa: E402
from gpu_util import DEV, dev_f, dev_h, dev_i, host, rel_err, rel_err_fp32   # noqa: E402

TOL16, TOL32 = 2e-2, 1e-5


def _progress(msg):
    print("[case] " + msg, flush=True)


# ------------------------------------------------------------------ sgd
@pytest.mark.parametrize("n", [0, 1, 7, 8, 1000, 4099, 262144 * 8 + 3])
def test_sgd_small_and_ragged(n):
    _progress("sgd n=%d" % n)
    g = synth.normal_f16(400, (n,), 1e-3)
    w0 = synth.normal_f32(401, (n,), 0.05)
    v0 = synth.normal_f32(402, (n,), 0.01)
    lr, mu, wd, s = 0.1, 0.9, 1e-4, 1.0 / 54000
    gd, wd_, vd = dev_h(g), dev_f(w0), dev_f(v0)
    lo = torch.zeros(max(n, 1), dtype=torch.float16, device=DEV)
    P.sgd_momentum_flat(n, gd, s, wd_, vd, lo, lr, mu, wd)
    w, v = w0.astype(np.float64), v0.astype(np.float64)
    low = O.sgd_momentum_flat(g.astype(np.float64), w, v, lr, mu, wd, s)
    if n:
        assert rel_err_fp32(host(wd_), w, 1e-3) <= TOL32 and rel_err_fp32(host(vd), v, 1e-3) <= TOL32
        # the half copy is decided from the FP32 weight: compare with the rounding of the GPU's own FP32 result
        assert np.array_equal(host(lo)[:n], O.round_binary16(host(wd_)))
        assert rel_err(host(lo)[:n], low) <= 2e-3


def test_sgd_full_size_100_steps():
    """Flat 25,557,032-element tail, 100 steps on the same gradient; parity after steps 1, 2, 100.

    Against the FP32 oracle (the paper's optimizer precision, same operation order) the result
    must be bit-identical; against the FP64 oracle within 1e-5 (elements that cancel to less
    than 1e-3 of the largest weight are measured against that floor)."""
    n = 25557032
    _progress("sgd full n=%d" % n)
    g = synth.normal_f16(400, (n,), 1e-3)
    w0 = synth.normal_f32(401, (n,), 0.05)
    lr, mu, wd, s = 0.1, 0.9, 1e-4, 1.0 / 54000
    gd, wdv, vd = dev_h(g), dev_f(w0), torch.zeros(n, dtype=torch.float32, device=DEV)
    lo = torch.empty(n, dtype=torch.float16, device=DEV)
    w, v = w0.astype(np.float32), np.zeros(n, np.float32)
    w64, v64 = w0.astype(np.float64), np.zeros(n, np.float64)
    g32, g64 = g.astype(np.float32), g.astype(np.float64)
    for step in range(1, 101):
        P.sgd_momentum_flat(n, gd, s, wdv, vd, lo, lr, mu, wd)
        O.sgd_momentum_flat(g32, w, v, np.float32(lr), np.float32(mu), np.float32(wd), np.float32(s), want_lowp=False)
        if step <= 2:
            O.sgd_momentum_flat(g64, w64, v64, float(np.float32(lr)), float(np.float32(mu)), float(np.float32(wd)),
                                float(np.float32(s)), want_lowp=False)
        if step in (1, 2, 100):
            gw, gv = host(wdv), host(vd)
            _progress("sgd step %d: max|w-w_fp32oracle| = %.3e" % (step, np.max(np.abs(gw - w))))
            assert np.array_equal(gw, w.astype(np.float64)) and np.array_equal(gv, v.astype(np.float64))
            if step <= 2:
                assert rel_err_fp32(gw, w64, 1e-3) <= TOL32 and rel_err_fp32(gv, v64, 1e-3) <= TOL32
    assert np.array_equal(host(lo), O.round_binary16(host(wdv)))


def test_sgd_no_lowp_and_errors():
    n = 1024
    g, w, v = dev_h(np.ones(n)), dev_f(np.ones(n)), dev_f(np.zeros(n))
    P.sgd_momentum_flat(n, g, 1.0, w, v, None, 0.5, 0.0, 0.0)
    assert np.allclose(host(w), 0.5)
    with pytest.raises(P.Rn50Error):
        P.sgd_momentum_flat(n, None, 1.0, w, v, None, 0.5, 0.0, 0.0)
    with pytest.raises(P.Rn50Error):
        P.sgd_momentum_flat(n, g, 1.0, w, v, None, 0.5, 0.0, 0.0, grad_dt=P.RN50_BF16)


# ------------------------------------------------------------------ LARS
def _lars_case(n, segments, seed, steps=1, wd=1e-4, s=1.0 / 1024, g_std=1.0):
    g = synth.normal_f16(seed, (n,), g_std)
    w0 = synth.normal_f32(seed + 1, (n,), 0.05)
    v0 = synth.normal_f32(seed + 2, (n,), 0.01)
    lr, mu, eta, eps = 0.5, 0.9, 0.01, 1e-6
    gd, wdv, vd = dev_h(g), dev_f(w0), dev_f(v0)
    lo = torch.full((max(n, 1),), 7.0, dtype=torch.float16, device=DEV)
    rates = torch.zeros(max(len(segments), 1), dtype=torch.float32, device=DEV)
    plan = P.LarsPlan(segments, DEV)
    w32, v32 = w0.copy(), v0.copy()
    w64, v64 = w0.astype(np.float64), v0.astype(np.float64)
    f = lambda x: float(np.float32(x))   # noqa: E731
    for step in range(steps):
        plan.step(gd, s, wdv, vd, lo, lr, mu, wd, eta, eps, rates)
        _, r32 = O.lars_momentum_flat(g.astype(np.float32), w32, v32, segments, np.float32(lr), np.float32(mu), np.float32(wd),
                                      np.float32(eta), np.float32(eps), np.float32(s), want_lowp=False)
        _, r64 = O.lars_momentum_flat(g.astype(np.float64), w64, v64, segments, f(lr), f(mu), f(wd), f(eta), f(eps), f(s),
                                      want_lowp=False)
        gw, gv, gr = host(wdv), host(vd), host(rates)[:len(segments)]
        if len(segments):
            # the layer rates: norms are summed in a different order than the oracle's, everything else is identical
            assert np.max(np.abs(gr - r64) / np.abs(r64)) <= TOL32, "rates step %d" % step
            assert np.max(np.abs(gr - r32.astype(np.float64)) / np.abs(r64)) <= TOL32
        if n:
            # FP32 oracle (the paper's optimizer precision, same operation order): 1e-5 with the usual floor.  Against
            # the FP64 oracle the FP32 rounding of v (which enters w undamped here: w -= v) is measured against 1e-2
            # of the largest element.
            assert rel_err_fp32(gw, w32.astype(np.float64), 1e-3) <= TOL32 and rel_err_fp32(gv, v32.astype(np.float64), 1e-3) <= TOL32, \
                "step %d" % step
            assert rel_err_fp32(gw, w64, 1e-2) <= TOL32 and rel_err_fp32(gv, v64, 1e-2) <= TOL32, "step %d" % step
    if n:
        covered = np.zeros(n, bool)
        for o, c, _ in segments:
            covered[o:o + c] = True
        gw, gv, glo = host(wdv), host(vd), host(lo)[:n]
        # outside every segment nothing is touched; inside, the half copy is the rounding of the GPU's own FP32 weight
        assert np.array_equal(gw[~covered], w0[~covered].astype(np.float64)) and np.array_equal(gv[~covered], v0[~covered].astype(np.float64))
        assert np.all(glo[~covered] == 7.0)
        assert np.array_equal(glo[covered], O.round_binary16(gw)[covered])
    plan.close()


@pytest.mark.parametrize("case", [
    (0, []), (8, [(0, 8, True)]), (64, [(0, 1, True), (8, 7, False), (16, 48, True)]),
    (5000, [(0, 2048, True), (2048, 2049, True), (4104, 1, False), (4112, 880, True)]),
    (2 ** 20 + 24, [(8, 2 ** 20 + 11, True), (0, 8, False)]),
    (70000, [(i * 1000, 999 - (i % 7), i % 3 != 0) for i in range(70)])])
def test_lars_small_and_ragged(case):
    n, segments = case
    _progress("lars n=%d nseg=%d" % (n, len(segments)))
    _lars_case(n, segments, 500, steps=2)


def test_lars_resnet50_layout_three_steps():
    """The flat 25,557,032-parameter buffer with the real segment table (161 tensors: filters and the FC weight with
    layer-wise scaling, BN scale / shift and the FC bias without), three steps on the same gradient."""
    cfg = P.make_config(32)
    lay = P.rn50_param_layout(cfg)
    segments = [(off, cnt, kind in (P.RN50_KIND_CONV, P.RN50_KIND_FCW)) for (kind, off, cnt, fan) in lay]
    n = P.rn50_param_count(cfg)
    assert n == 25557032 and len(segments) == 161
    _progress("lars full n=%d" % n)
    _lars_case(n, segments, 510, steps=3, s=1.0 / 54000, g_std=1e-3)


def test_lars_degenerate_norms_and_errors():
    # zero gradient / zero weights: rate 1
    n = 4096
    plan = P.LarsPlan([(0, 2048, True), (2048, 2048, True)], DEV)
    g = np.zeros(n, np.float16); g[2048:] = 0.5
    w0 = np.ones(n, np.float32); w0[2048:] = 0
    gd, wdv, vd = dev_h(g), dev_f(w0), torch.zeros(n, dtype=torch.float32, device=DEV)
    rates = torch.zeros(2, dtype=torch.float32, device=DEV)
    plan.step(gd, 1.0, wdv, vd, None, 0.5, 0.0, 0.0, 0.01, 0.0, rates)
    assert np.array_equal(host(rates), [1.0, 1.0])
    assert np.all(host(wdv)[:2048] == 1.0) and np.all(host(wdv)[2048:] == -0.25)
    plan.close()
    for bad in ([(4, 8, True)], [(0, 16, True), (8, 16, False)]):      # misaligned offset, overlap
        with pytest.raises(P.Rn50Error):
            P.LarsPlan(bad, DEV)
    plan = P.LarsPlan([(0, 64, True)], DEV)
    x = torch.zeros(64, dtype=torch.float32, device=DEV)
    with pytest.raises(P.Rn50Error):
        plan.step(None, 1.0, x, x.clone(), None, 0.1, 0.9, 0.0, 0.01, 1e-6)
    with pytest.raises(P.Rn50Error):
        plan.step(x.half(), 1.0, x, x.clone(), None, 0.1, 0.9, 0.0, 0.0, 1e-6)     # eta must be positive
    plan.close()


# ------------------------------------------------------------------ loss
@pytest.mark.parametrize("batch,classes", [(1, 2), (2, 10), (32, 1000), (16, 1000), (128, 1000), (37, 1001), (3, 4096)])
def test_ls_xent(batch, classes):
    _progress("ls_xent batch=%d classes=%d" % (batch, classes))
    z = synth.normal_f32(500 + batch, (batch, classes), 3.0)
    lab = synth.labels(501 + batch, batch, classes)
    scale = 128.0 / batch
    zd, ld = dev_f(z), dev_i(lab)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    per = torch.zeros(batch, dtype=torch.float32, device=DEV)
    dz = torch.zeros(batch, classes, dtype=torch.float16, device=DEV)
    P.ls_xent_fwd_bwd(batch, classes, zd, ld, 0.1, scale, loss, per, dz)
    rl, rper, rdz = O.ls_xent_fwd_bwd(z.astype(np.float64), lab, 0.1, scale)
    assert rel_err_fp32(host(loss), [rl]) <= TOL32
    assert rel_err_fp32(host(per), rper) <= TOL32
    assert rel_err(host(dz), rdz) <= TOL16
    # deterministic, and loss_per_sample may be NULL
    loss2 = torch.zeros(1, dtype=torch.float32, device=DEV)
    P.ls_xent_fwd_bwd(batch, classes, zd, ld, 0.1, scale, loss2, None, dz)
    assert host(loss2)[0] == host(loss)[0]


def test_ls_xent_closed_forms_on_gpu():
    k = 1000
    z = dev_f(np.full((32, k), 0.37))
    lab = dev_i(synth.labels(7, 32, k))
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    dz = torch.zeros(32, k, dtype=torch.float16, device=DEV)
    P.ls_xent_fwd_bwd(32, k, z, lab, 0.1, 1.0, loss, None, dz)
    assert abs(host(loss)[0] - np.log(k)) <= TOL32 * np.log(k)
    big = dev_f(synth.normal_f32(8, (32, k), 3000.0))           # no overflow with huge logits
    P.ls_xent_fwd_bwd(32, k, big, lab, 0.1, 1.0, loss, None, dz)
    assert np.isfinite(host(loss)[0]) and np.all(np.isfinite(host(dz)))
    with pytest.raises(P.Rn50Error):
        P.ls_xent_fwd_bwd(0, k, z, lab, 0.1, 1.0, loss, None, dz)


# ------------------------------------------------------------------ batch norm
BN_CASES = [  # m, c, relu, residual
    (1, 8, True, False), (50, 8, False, False), (2 * 56 * 56, 64, True, False), (2 * 56 * 56, 256, True, True),
    (2 * 56 * 56 + 5, 256, False, False), (3 * 7 * 7, 2048, True, True), (1000, 512, True, False),
    (3001, 128, True, True), (77, 4096, True, False), (4 * 112 * 112, 64, True, False)]


@pytest.mark.parametrize("m,c,relu,res", BN_CASES)
def test_bn_relu_fwd_bwd(m, c, relu, res):
    _progress("bn m=%d c=%d relu=%d res=%d" % (m, c, relu, res))
    x = synth.normal_f16(600, (m, c)) * 1.5
    x = (x + synth.normal_f32(601, (c,), 0.7)).astype(np.float16).astype(np.float32)
    gamma = 1.0 + synth.normal_f32(602, (c,), 0.2)
    beta = synth.normal_f32(603, (c,), 0.3)
    r = synth.normal_f16(604, (m, c)) if res else None
    dy = synth.normal_f16(605, (m, c), 0.05)
    d = P.make_bn_desc(m, c, 1e-5, relu, res)
    xd, gd, bd = dev_h(x), dev_f(gamma), dev_f(beta)
    rd = dev_h(r) if res else None
    y = torch.zeros(m, c, dtype=torch.float16, device=DEV)
    mean = torch.zeros(c, dtype=torch.float32, device=DEV)
    invstd = torch.zeros(c, dtype=torch.float32, device=DEV)
    P.bn_relu_fwd(d, xd, gd, bd, rd, y, mean, invstd)
    f64 = np.float64
    ry, rmean, rinv, _ = O.bn_relu_fwd(x.astype(f64), gamma.astype(f64), beta.astype(f64), 1e-5, relu,
                                       r.astype(f64) if res else None)
    if m > 1:
        assert rel_err_fp32(host(invstd), rinv) <= 1e-4
    assert np.max(np.abs(host(mean) - rmean)) <= 1e-5 * max(1.0, np.max(np.abs(rmean)))
    assert rel_err(host(y), ry) <= TOL16
    # backward, fed with the oracle's (rounded) forward output and statistics
    y16 = O.round_binary16(ry)
    yd = dev_h(y16)
    dx = torch.zeros(m, c, dtype=torch.float16, device=DEV)
    dres = torch.zeros(m, c, dtype=torch.float16, device=DEV) if res else None
    dg = torch.zeros(c, dtype=torch.float16, device=DEV)
    db = torch.zeros(c, dtype=torch.float16, device=DEV)
    P.bn_relu_bwd(d, dev_h(dy), xd, yd if relu else None, gd, dev_f(rmean), dev_f(rinv), dx, dres, dg, db)
    rdx, rdres, rdg, rdb = O.bn_relu_bwd(dy.astype(f64), x.astype(f64), y16, gamma.astype(f64),
                                         rmean.astype(np.float32).astype(f64), rinv.astype(np.float32).astype(f64),
                                         relu, res)
    assert rel_err(host(dx), rdx) <= TOL16
    assert rel_err(host(dg), rdg) <= TOL16 and rel_err(host(db), rdb) <= TOL16
    if res:
        assert np.array_equal(host(dres), rdres)          # pure masking of FP16 values: exact


@pytest.mark.parametrize("m_a,m_b,c,relu,res", [(700, 324, 64, True, True), (2 * 28 * 28, 3 * 28 * 28, 128, True, False),
                                                 (5, 3000, 512, False, False), (1, 1, 8, True, False)])
def test_bn_split_at_exchange_points_two_way(m_a, m_b, c, relu, res):
    """Synchronised batch norm built from the four split entry points: two local batches ("two GPUs"), moments
    averaged by rows and backward sums added on the host, must match the oracle's batch norm over the union."""
    _progress("bn split m=%d+%d c=%d relu=%d res=%d" % (m_a, m_b, c, relu, res))
    m = m_a + m_b
    x = synth.normal_f16(620, (m, c)) * 1.5
    x = (x + synth.normal_f32(621, (c,), 0.7)).astype(np.float16).astype(np.float32)
    x[m_a:] += np.float32(0.5)                                  # the two halves have different statistics
    x = x.astype(np.float16).astype(np.float32)
    gamma, beta = 1.0 + synth.normal_f32(622, (c,), 0.2), synth.normal_f32(623, (c,), 0.3)
    r = synth.normal_f16(624, (m, c)) if res else None
    dy = synth.normal_f16(625, (m, c), 0.05)
    f64 = np.float64
    ry, rmean, rinv, rsq = O.bn_relu_fwd(x.astype(f64), gamma.astype(f64), beta.astype(f64), 1e-5, relu, r.astype(f64) if res else None)
    parts = [(0, m_a), (m_a, m)]
    gd, bd = dev_f(gamma), dev_f(beta)
    descs, xs, moms = [], [], []
    for lo, hi in parts:
        d = P.make_bn_desc(hi - lo, c, 1e-5, relu, res)
        xd = dev_h(x[lo:hi])
        mom = torch.zeros(2 * c, dtype=torch.float32, device=DEV)
        P.bn_batch_moments(d, xd, mom)
        ma, qa = O.bn_moments(x[lo:hi].astype(f64))
        assert np.max(np.abs(host(mom)[:c] - ma)) <= 1e-5 * max(1.0, np.max(np.abs(ma)))
        assert rel_err_fp32(host(mom)[c:], qa) <= 1e-5
        descs.append(d); xs.append(xd); moms.append(host(mom))
    comb = (moms[0] * m_a + moms[1] * m_b) / m                                 # what an all-reduce would deliver
    assert np.max(np.abs(comb[:c] - rmean)) <= 1e-5 * max(1.0, np.max(np.abs(rmean))) and rel_err_fp32(comb[c:], rsq) <= 1e-5
    combd = dev_f(comb.astype(np.float32))
    ys, means, invs = [], [], []
    for (lo, hi), d, xd in zip(parts, descs, xs):
        y = torch.zeros(hi - lo, c, dtype=torch.float16, device=DEV)
        mean, inv = torch.zeros(c, dtype=torch.float32, device=DEV), torch.zeros(c, dtype=torch.float32, device=DEV)
        P.bn_relu_fwd_from_moments(d, xd, gd, bd, dev_h(r[lo:hi]) if res else None, y, combd, mean, inv)
        ys.append(host(y)); means.append(mean); invs.append(inv)
    if m > 2:
        assert rel_err_fp32(host(invs[0]), rinv) <= 1e-4
        assert rel_err(np.concatenate(ys), ry) <= TOL16
    # backward with the oracle's rounded forward output and statistics
    y16 = O.round_binary16(ry)
    m32, i32 = rmean.astype(np.float32), rinv.astype(np.float32)
    rdx, rdres, rdg, rdb = O.bn_relu_bwd(dy.astype(f64), x.astype(f64), y16, gamma.astype(f64), m32.astype(f64), i32.astype(f64), relu, res)
    md, idv = dev_f(m32), dev_f(i32)
    sums = []
    for (lo, hi), d, xd in zip(parts, descs, xs):
        sm = torch.zeros(2 * c, dtype=torch.float32, device=DEV)
        P.bn_relu_bwd_sums(d, dev_h(dy[lo:hi]), xd, dev_h(y16[lo:hi]) if relu else None, md, idv, sm)
        sums.append(host(sm))
    tot = sums[0] + sums[1]
    assert rel_err_fp32(tot[:c], rdb, 1e-3) <= 1e-4 and rel_err_fp32(tot[c:], rdg, 1e-3) <= 1e-4
    totd = dev_f(tot.astype(np.float32))
    dxs, drs = [], []
    for (lo, hi), d, xd in zip(parts, descs, xs):
        dx = torch.zeros(hi - lo, c, dtype=torch.float16, device=DEV)
        dres = torch.zeros(hi - lo, c, dtype=torch.float16, device=DEV) if res else None
        P.bn_relu_bwd_from_sums(d, dev_h(dy[lo:hi]), xd, dev_h(y16[lo:hi]) if relu else None, gd, md, idv, totd, m, dx, dres)
        dxs.append(host(dx)); drs.append(host(dres) if res else None)
    assert rel_err(np.concatenate(dxs), rdx) <= TOL16
    if res:
        assert np.array_equal(np.concatenate(drs), rdres)
    with pytest.raises(P.Rn50Error):                                   # the total row count cannot be below the local one
        P.bn_relu_bwd_from_sums(descs[1], dev_h(dy[m_a:]), xs[1], dev_h(y16[m_a:]) if relu else None, gd, md, idv, totd, m_b - 1,
                                torch.zeros(m_b, c, dtype=torch.float16, device=DEV),
                                torch.zeros(m_b, c, dtype=torch.float16, device=DEV) if res else None)


def test_bn_large_mean_channel_and_determinism():
    m, c = 5000, 64
    x = synth.normal_f16(610, (m, c))
    x[:, 3] = (100.0 + x[:, 3]).astype(np.float16).astype(np.float32)     # mean = 100 sigma
    d = P.make_bn_desc(m, c, 1e-5, True, False)
    xd = dev_h(x)
    g, b = dev_f(np.ones(c)), dev_f(np.zeros(c))
    outs = []
    for _ in range(2):
        y = torch.zeros(m, c, dtype=torch.float16, device=DEV)
        mean = torch.zeros(c, dtype=torch.float32, device=DEV)
        invstd = torch.zeros(c, dtype=torch.float32, device=DEV)
        P.bn_relu_fwd(d, xd, g, b, None, y, mean, invstd)
        outs.append((host(y), host(mean), host(invstd)))
    assert all(np.array_equal(a, b_) for a, b_ in zip(outs[0], outs[1]))
    _, rmean, rinv, _ = O.bn_relu_fwd(x.astype(np.float64), np.ones(c), np.zeros(c), 1e-5, True)
    assert rel_err_fp32(outs[0][2], rinv) <= 1e-4
    # mean: absolute error measured against the channel's scale (sigma = 1 here, or |mean| if larger)
    assert np.max(np.abs(outs[0][1] - rmean) / np.maximum(np.abs(rmean), 1.0)) <= 1e-5


def test_bn_error_paths():
    d = P.make_bn_desc(10, 12)                      # c not a multiple of 8
    t = torch.zeros(256, dtype=torch.float16, device=DEV)
    f = torch.zeros(64, dtype=torch.float32, device=DEV)
    with pytest.raises(P.Rn50Error):
        P.bn_relu_fwd(d, t, f, f, None, t, f, f, ws=torch.zeros(1 << 20, dtype=torch.uint8, device=DEV))
    d = P.make_bn_desc(10, 16)
    with pytest.raises(P.Rn50Error):                # workspace too small
        P.bn_relu_fwd(d, t, f, f, None, t, f, f, ws=torch.zeros(16, dtype=torch.uint8, device=DEV))
