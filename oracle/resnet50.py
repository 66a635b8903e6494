"""Oracle of the whole per-GPU training iteration -- TEST INFRASTRUCTURE ONLY.

Chains the plain-C definitions (oracle/__init__.py) over a ResNet-50 v1.5 style
network: forward, label-smoothed softmax cross-entropy, backward, momentum SGD
on the flat parameter buffer (paper Sec. 2: per-GPU forward/backward followed by
the update; Sec. 3.2: ResNet-50, FP16 forward/backward with FP32 batch-norm
statistics and an FP32 optimizer).

The network description and the flat parameter order are written here
independently of the HIP library; a test checks that the two agree.

Topology: optional stem (7x7/2 conv 3->64 pad 3, BN, ReLU, 3x3/2 max-pool pad 1),
then stages of bottleneck blocks (1x1 -> 3x3 -> 1x1, widths w/w/4w, the 3x3
carries the stride), a 1x1 projection shortcut (+BN, no ReLU) on the first
block of every stage, one ReLU after the residual add, global average pool, FC.

Flat parameter order (network order): for every conv: filter KRSC, then its BN
gamma, then its BN beta; inside a block conv1, conv2, conv3, projection; after
the last block the FC weight [classes, C] and last the FC bias.

"lowp" mode rounds to binary16 at exactly the places where the mixed-precision
path stores a tensor: every activation, every activation gradient, the FP16
copy of conv/FC weights, the flat gradient.  Statistics, logits, loss and the
update stay in the working precision.
"""
import numpy as np

import oracle as O


class Segment:
    def __init__(self, name, kind, shape, offset, fan_in):
        self.name, self.kind, self.shape, self.offset, self.fan_in = name, kind, tuple(shape), offset, fan_in
        self.count = int(np.prod(shape))


KIND_CONV, KIND_GAMMA, KIND_BETA, KIND_FCW, KIND_FCB = 0, 1, 2, 3, 4


class Net:
    """Static description: convs, blocks and the flat parameter layout."""

    def __init__(self, batch, in_hw, has_stem=True, blocks=(3, 4, 6, 3), base_width=64, classes=1000):
        self.batch, self.in_hw, self.has_stem = batch, tuple(in_hw), has_stem
        self.blocks, self.base_width, self.classes = tuple(blocks), base_width, classes
        self.segments = []
        self._off = 0
        self.convs = {}          # name -> dict(cin, cout, r, stride, pad)
        self.block_list = []     # dicts: name, cin, width, cout, stride, proj
        if has_stem:
            self._add_conv("stem", 3, base_width, 7, 2, 3)
        cin = base_width
        for si, nb in enumerate(self.blocks):
            width = base_width << si
            cout = 4 * width
            for bi in range(nb):
                stride = 2 if (bi == 0 and si > 0) else 1
                name = "s%db%d" % (si + 1, bi)
                proj = bi == 0
                self._add_conv(name + "c1", cin, width, 1, 1, 0)
                self._add_conv(name + "c2", width, width, 3, stride, 1)
                self._add_conv(name + "c3", width, cout, 1, 1, 0)
                if proj:
                    self._add_conv(name + "p", cin, cout, 1, stride, 0)
                self.block_list.append(dict(name=name, cin=cin, width=width, cout=cout, stride=stride, proj=proj))
                cin = cout
        self.feat = cin
        self._add("fc.w", KIND_FCW, (classes, cin), cin)
        self._add("fc.b", KIND_FCB, (classes,), cin)
        self.param_count = self._off
        self.seg = {s.name: s for s in self.segments}

    def _add(self, name, kind, shape, fan_in):
        s = Segment(name, kind, shape, self._off, fan_in)
        self.segments.append(s)
        self._off += s.count

    def _add_conv(self, name, cin, cout, r, stride, pad):
        self.convs[name] = dict(cin=cin, cout=cout, r=r, stride=stride, pad=pad)
        self._add(name + ".w", KIND_CONV, (cout, r, r, cin), cin * r * r)
        self._add(name + ".gamma", KIND_GAMMA, (cout,), 0)
        self._add(name + ".beta", KIND_BETA, (cout,), 0)

    def view(self, flat, name):
        s = self.seg[name]
        return flat[s.offset:s.offset + s.count].reshape(s.shape)


def _make_ctx(net, master_w, lowp, dtype):
    st = (lambda a: O.round_binary16(a)) if lowp else (lambda a: a)
    w_master = np.asarray(master_w, dtype)
    w_fwd = st(w_master)                     # FP16 copy used by conv / FC weights

    def P(name, low=True):
        return net.view(w_fwd if low else w_master, name)
    return st, w_master, P


def forward_ref(net, images, master_w, bn_eps=1e-5, lowp=True, dtype=np.float64):
    """Forward pass.  Returns the dict t of every stored tensor:
    '<conv>.in', '<conv>.conv', '<conv>.out', '<conv>.mean', '<conv>.invstd', 'pool.out',
    '<block>.in', 'feat', 'logits'."""
    st, _, P = _make_ctx(net, master_w, lowp, dtype)
    t = {}

    def conv_bn_fwd(name, x, relu, residual=None):
        cv = net.convs[name]
        t[name + ".in"] = x
        c = st(O.conv_fwd(x, P(name + ".w"), cv["stride"], cv["pad"]))
        t[name + ".conv"] = c
        y, mean, invstd, _ = O.bn_relu_fwd(c, P(name + ".gamma", False), P(name + ".beta", False),
                                           bn_eps, relu, residual)
        y = st(y)
        t[name + ".mean"], t[name + ".invstd"], t[name + ".out"] = mean, invstd, y
        return y

    x = st(np.asarray(images, dtype))
    if net.has_stem:
        y = conv_bn_fwd("stem", x, True)
        x = st(O.maxpool_fwd(y, 3, 2, 1))
        t["pool.out"] = x
    for b in net.block_list:
        n = b["name"]
        t[n + ".in"] = x
        a = conv_bn_fwd(n + "c1", x, True)
        a = conv_bn_fwd(n + "c2", a, True)
        sc = conv_bn_fwd(n + "p", x, False) if b["proj"] else x
        x = conv_bn_fwd(n + "c3", a, True, residual=sc)
    feat = st(O.avgpool_fwd(x))
    t["feat"] = feat
    t["logits"] = O.fc_fwd(feat, P("fc.w"), P("fc.b", False))
    return t


def backward_ref(net, t, labels, master_w, ls_eps=0.1, loss_scale=1.0, lowp=True, dtype=np.float64):
    """Loss and backward pass from a dict t of forward tensors (forward_ref's own, or tensors
    produced elsewhere with the same names: '<conv>.in' may be omitted for convs whose input is a
    block input, in which case '<block>.in' is used).  Adds '<conv>.dconv', '<block>.dout',
    'dlogits', 'pool.dout' to t.  Returns loss, loss_per_sample, flat gradient."""
    st, _, P = _make_ctx(net, master_w, lowp, dtype)
    grad = np.zeros(net.param_count, dtype)

    def G(name, val):
        s = net.seg[name]
        grad[s.offset:s.offset + s.count] = st(np.asarray(val, dtype)).reshape(-1)

    def conv_bn_bwd(name, dy, relu, want_dres, need_dx=True):
        cv = net.convs[name]
        x, c, y = t[name + ".in"], t[name + ".conv"], t[name + ".out"]
        dc, dres, dgamma, dbeta = O.bn_relu_bwd(dy, c, y, P(name + ".gamma", False), t[name + ".mean"],
                                                t[name + ".invstd"], relu, want_dres)
        dc = st(dc)
        t[name + ".dconv"] = dc
        if dres is not None:
            dres = st(dres)
        G(name + ".gamma", dgamma)
        G(name + ".beta", dbeta)
        G(name + ".w", O.conv_wgrad(x, dc, net.seg[name + ".w"].shape, cv["stride"], cv["pad"]))
        dx = O.conv_dgrad(dc, P(name + ".w"), x.shape, cv["stride"], cv["pad"]) if need_dx else None
        return dx, dres

    logits, feat = t["logits"], t["feat"]
    bsz = logits.shape[0]
    loss, per, dz = O.ls_xent_fwd_bwd(logits, labels, ls_eps, loss_scale / bsz)
    dz = st(dz)
    t["dlogits"] = dz
    dwt, db, da = O.fc_bwd(feat, P("fc.w"), dz)
    G("fc.w", dwt)
    G("fc.b", db)
    da = st(da)
    last = net.block_list[-1]["name"] + "c3"
    dx = st(O.avgpool_bwd(da, t[last + ".out"].shape[1:3]))
    first = net.block_list[0]["name"]
    for b in reversed(net.block_list):
        n = b["name"]
        need_in = net.has_stem or n != first
        t[n + ".dout"] = dx
        d3, dres = conv_bn_bwd(n + "c3", dx, True, True)
        d2, _ = conv_bn_bwd(n + "c2", st(d3), True, False)
        d1, _ = conv_bn_bwd(n + "c1", st(d2), True, False, need_dx=need_in)
        if b["proj"]:
            dp, _ = conv_bn_bwd(n + "p", dres, False, False, need_dx=need_in)
            dx = st(d1 + st(dp)) if need_in else None
        else:
            dx = st(d1 + dres)
    if net.has_stem:
        t["pool.dout"] = dx
        dstem = st(O.maxpool_bwd(t["stem.out"], dx, 3, 2, 1))
        conv_bn_bwd("stem", dstem, True, False, need_dx=False)
    return loss, per, grad


def step_ref(net, images, labels, master_w, momentum, lr, mu, wd, ls_eps=0.1, bn_eps=1e-5,
             loss_scale=1.0, lowp=True, dtype=np.float64, update=True):
    """One training iteration.  images NHWC, labels int, master_w/momentum flat arrays.

    Returns a dict with every stored tensor ('t'), the loss, the flat gradient
    (scaled by loss_scale, rounded to binary16 in lowp mode) and the updated
    w / v / w_lowp.  Inputs are not modified.
    """
    t = forward_ref(net, images, master_w, bn_eps, lowp, dtype)
    loss, per, grad = backward_ref(net, t, labels, master_w, ls_eps, loss_scale, lowp, dtype)
    out = dict(t=t, loss=loss, loss_per_sample=per, grad=grad)
    if update:
        w_new = np.asarray(master_w, dtype).copy()
        v_new = np.asarray(momentum, dtype).copy()
        out["w_lowp"] = O.sgd_momentum_flat(grad, w_new, v_new, lr, mu, wd, 1.0 / loss_scale)
        out["w"], out["v"] = w_new, v_new
    return out
