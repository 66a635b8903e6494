"""Thin Python binding of librn50.so (hand-written HIP for gfx950).

Argument marshalling only: torch tensors supply device memory and the current
stream; every step of the path runs inside the library's kernels.  Function
names and argument order follow include/rn50.h.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librn50.so")

RN50_F16, RN50_BF16 = 0, 1
CONV_FWD, CONV_DGRAD, CONV_WGRAD = 0, 1, 2
KIND_CONV, KIND_GAMMA, KIND_BETA, KIND_FCW, KIND_FCB = 0, 1, 2, 3, 4


class Rn50Error(RuntimeError):
    pass


class conv_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("n", "h", "w", "c", "k", "r", "s", "stride", "pad", "dt")]


class bn_desc(ctypes.Structure):
    _fields_ = [("m", ctypes.c_longlong), ("c", ctypes.c_int), ("eps", ctypes.c_float), ("relu", ctypes.c_int),
                ("has_residual", ctypes.c_int), ("dt", ctypes.c_int)]


class rn50_config(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int), ("image_h", ctypes.c_int), ("image_w", ctypes.c_int),
                ("has_stem", ctypes.c_int), ("num_stages", ctypes.c_int), ("blocks", ctypes.c_int * 4),
                ("base_width", ctypes.c_int), ("classes", ctypes.c_int), ("dt", ctypes.c_int),
                ("bn_eps", ctypes.c_float), ("ls_eps", ctypes.c_float), ("loss_scale", ctypes.c_float),
                ("keep_grads", ctypes.c_int)]


class rn50_profile_entry(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("launches", ctypes.c_longlong), ("total_ms", ctypes.c_double),
                ("flops", ctypes.c_double), ("bytes", ctypes.c_double), ("side_launches", ctypes.c_longlong)]


RN50_KIND_CONV, RN50_KIND_GAMMA, RN50_KIND_BETA, RN50_KIND_FCW, RN50_KIND_FCB = 0, 1, 2, 3, 4


class rn50_hparams(ctypes.Structure):
    """lars_eta == 0: momentum SGD; lars_eta > 0: LARS with momentum (coefficient lars_eta, lars_eps)."""
    _fields_ = [("lr", ctypes.c_float), ("momentum", ctypes.c_float), ("wd", ctypes.c_float),
                ("grad_scale", ctypes.c_float), ("lars_eta", ctypes.c_float), ("lars_eps", ctypes.c_float)]


class rn50_lars_segment(ctypes.Structure):
    _fields_ = [("offset", ctypes.c_size_t), ("count", ctypes.c_size_t), ("use_lars", ctypes.c_int)]


_lib = None
_vp, _sz, _i, _f = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float

_SIGNATURES = {
    "rn50_status_string": (ctypes.c_char_p, [_i]),
    "rn50_last_hip_error": (_i, []),
    "conv_workspace_bytes": (_sz, [ctypes.POINTER(conv_desc), _i]),
    "conv_fwd": (_i, [ctypes.POINTER(conv_desc), _vp, _vp, _vp, _vp, _sz, _vp]),
    "conv_dgrad": (_i, [ctypes.POINTER(conv_desc), _vp, _vp, _vp, _vp, _sz, _vp]),
    "conv_wgrad": (_i, [ctypes.POINTER(conv_desc), _vp, _vp, _vp, _vp, _sz, _vp]),
    "rn50_conv_variant_count": (_i, [_i]),
    "rn50_conv_variant_applies": (_i, [ctypes.POINTER(conv_desc), _i, _i]),
    "conv_fwd_variant": (_i, [ctypes.POINTER(conv_desc), _vp, _vp, _vp, _vp, _sz, _i, _vp]),
    "conv_dgrad_variant": (_i, [ctypes.POINTER(conv_desc), _vp, _vp, _vp, _vp, _sz, _i, _vp]),
    "conv_wgrad_variant": (_i, [ctypes.POINTER(conv_desc), _vp, _vp, _vp, _vp, _sz, _i, _vp]),
    "bn_workspace_bytes": (_sz, [ctypes.POINTER(bn_desc)]),
    "bn_relu_fwd": (_i, [ctypes.POINTER(bn_desc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_relu_fwd_static": (_i, [ctypes.POINTER(bn_desc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "bn_relu_bwd": (_i, [ctypes.POINTER(bn_desc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_batch_moments": (_i, [ctypes.POINTER(bn_desc), _vp, _vp, _vp, _sz, _vp]),
    "bn_relu_fwd_from_moments": (_i, [ctypes.POINTER(bn_desc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "bn_relu_bwd_sums": (_i, [ctypes.POINTER(bn_desc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_relu_bwd_from_sums": (_i, [ctypes.POINTER(bn_desc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_longlong, _vp, _vp, _vp]),
    "ls_xent_fwd_bwd": (_i, [_i, _i, _vp, _vp, _f, _f, _vp, _vp, _vp, _i, _vp]),
    "sgd_momentum_flat": (_i, [_sz, _vp, _i, _f, _vp, _vp, _vp, _f, _f, _f, _vp]),
    "lars_workspace_bytes": (_sz, [ctypes.POINTER(rn50_lars_segment), _i]),
    "lars_plan_create": (_i, [ctypes.POINTER(_vp), ctypes.POINTER(rn50_lars_segment), _i, _vp, _sz]),
    "lars_plan_destroy": (None, [_vp]),
    "lars_momentum_flat": (_i, [_vp, _vp, _i, _f, _vp, _vp, _vp, _f, _f, _f, _f, _f, _vp, _vp]),
    "rn50_sched_lr_b": (ctypes.c_double, [ctypes.c_double]),
    "rn50_sched_noise_scale_b": (ctypes.c_double, [ctypes.c_double]),
    "rn50_sched_momentum_b": (ctypes.c_double, [ctypes.c_double, ctypes.c_double]),
    "rn50_sched_batch": (_i, [_i, ctypes.c_double, ctypes.POINTER(_i), ctypes.POINTER(_i)]),
    "rn50_param_count": (_sz, [ctypes.POINTER(rn50_config)]),
    "rn50_num_segments": (_i, [ctypes.POINTER(rn50_config)]),
    "rn50_param_layout": (_i, [ctypes.POINTER(rn50_config), _i, ctypes.POINTER(_sz), ctypes.POINTER(_sz),
                               ctypes.POINTER(_i), ctypes.POINTER(_i)]),
    "rn50_workspace_bytes": (_sz, [ctypes.POINTER(rn50_config)]),
    "rn50_create": (_i, [ctypes.POINTER(_vp), ctypes.POINTER(rn50_config), _vp, _sz]),
    "rn50_destroy": (None, [_vp]),
    "rn50_cast_params": (_i, [_sz, _vp, _vp, _i, _vp]),
    "rn50_step": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.POINTER(rn50_hparams), _vp, _vp]),
    "rn50_profile_begin": (_i, []),
    "rn50_profile_end": (_i, [ctypes.POINTER(rn50_profile_entry), _i, ctypes.POINTER(_i)]),
    "rn50_autotune": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "rn50_get_tuning": (_i, [_vp, ctypes.POINTER(_i), _i]),
    "rn50_set_tuning": (_i, [_vp, ctypes.POINTER(_i), _i]),
    "rn50_tuning_report": (_sz, [_vp, ctypes.c_char_p, _sz]),
    "rn50_tensor": (_i, [_vp, ctypes.c_char_p, ctypes.POINTER(_vp), ctypes.POINTER(_sz), ctypes.POINTER(_i)]),
    "rn50_probe_mfma": (_i, [_i, _i, _vp, _vp]),
    "rn50_probe_tile_load": (_i, [_vp, _sz, _i, _i, _i, _i, _vp, _vp]),
    "rn50_probe_copy": (_i, [_vp, _vp, _sz, _vp]),
    "rn50_probe_empty": (_i, [_i, _vp]),
}
EXPORTS = tuple(_SIGNATURES)


def lib():
    """Load librn50.so (built by paper_1811_05233_amd/build.py).  Raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise Rn50Error("librn50.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        l = ctypes.CDLL(LIB_PATH)
        missing = []
        for name, (res, args) in _SIGNATURES.items():
            try:
                fn = getattr(l, name)
            except AttributeError:
                missing.append(name)
                continue
            fn.restype, fn.argtypes = res, args
        if missing:
            raise Rn50Error("librn50.so lacks %s: rebuild it" % ", ".join(missing))
        _lib = l
    return _lib


def _check(rc, what):
    if rc != 0:
        l = lib()
        msg = l.rn50_status_string(rc).decode()
        if rc == -6:
            msg += " (hipError %d)" % l.rn50_last_hip_error()
        raise Rn50Error("%s failed: %s" % (what, msg))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(nbytes, like):
    import torch
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=like.device)


# ------------------------------------------------------------------ kernels
def make_conv_desc(n, h, w, c, k, r, s, stride, pad, dt=RN50_F16):
    return conv_desc(n, h, w, c, k, r, s, stride, pad, dt)


def conv_workspace_bytes(d, which):
    return int(lib().conv_workspace_bytes(ctypes.byref(d), which))


def conv_variant_count(which):
    return int(lib().rn50_conv_variant_count(which))


def conv_fwd(d, x, w, y, ws=None, variant=None):
    ws = ws if ws is not None else _ws(conv_workspace_bytes(d, CONV_FWD), x)
    if variant is None:
        rc = lib().conv_fwd(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), _ptr(ws), ws.numel(), _stream())
    else:
        rc = lib().conv_fwd_variant(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), _ptr(ws), ws.numel(), int(variant), _stream())
    _check(rc, "conv_fwd")
    return y


def conv_dgrad(d, dy, w, dx, ws=None, variant=None):
    ws = ws if ws is not None else _ws(conv_workspace_bytes(d, CONV_DGRAD), dy)
    if variant is None:
        rc = lib().conv_dgrad(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(dx), _ptr(ws), ws.numel(), _stream())
    else:
        rc = lib().conv_dgrad_variant(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(dx), _ptr(ws), ws.numel(), int(variant), _stream())
    _check(rc, "conv_dgrad")
    return dx


def conv_wgrad(d, x, dy, dw, ws=None, variant=None):
    ws = ws if ws is not None else _ws(conv_workspace_bytes(d, CONV_WGRAD), x)
    if variant is None:
        rc = lib().conv_wgrad(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(ws), ws.numel(), _stream())
    else:
        rc = lib().conv_wgrad_variant(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(ws), ws.numel(), int(variant), _stream())
    _check(rc, "conv_wgrad")
    return dw


def make_bn_desc(m, c, eps=1e-5, relu=True, has_residual=False, dt=RN50_F16):
    return bn_desc(m, c, eps, int(relu), int(has_residual), dt)


def bn_workspace_bytes(d):
    return int(lib().bn_workspace_bytes(ctypes.byref(d)))


def bn_relu_fwd(d, x, gamma, beta, residual, y, save_mean, save_invstd, ws=None):
    ws = ws if ws is not None else _ws(bn_workspace_bytes(d), x)
    _check(lib().bn_relu_fwd(ctypes.byref(d), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(residual), _ptr(y),
                             _ptr(save_mean), _ptr(save_invstd), _ptr(ws), ws.numel(), _stream()), "bn_relu_fwd")
    return y


def bn_relu_fwd_static(d, x, gamma, beta, residual, y, save_mean, save_invstd):
    """bn_relu_fwd on the library's static device scratch (no workspace, no allocation; c <= 256)."""
    _check(lib().bn_relu_fwd_static(ctypes.byref(d), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(residual), _ptr(y),
                                    _ptr(save_mean), _ptr(save_invstd), _stream()), "bn_relu_fwd_static")
    return y


def bn_relu_bwd(d, dy, x, y, gamma, save_mean, save_invstd, dx, dresidual, dgamma, dbeta, ws=None):
    ws = ws if ws is not None else _ws(bn_workspace_bytes(d), x)
    _check(lib().bn_relu_bwd(ctypes.byref(d), _ptr(dy), _ptr(x), _ptr(y), _ptr(gamma), _ptr(save_mean),
                             _ptr(save_invstd), _ptr(dx), _ptr(dresidual), _ptr(dgamma), _ptr(dbeta),
                             _ptr(ws), ws.numel(), _stream()), "bn_relu_bwd")
    return dx


def bn_batch_moments(d, x, moments, ws=None):
    ws = ws if ws is not None else _ws(bn_workspace_bytes(d), x)
    _check(lib().bn_batch_moments(ctypes.byref(d), _ptr(x), _ptr(moments), _ptr(ws), ws.numel(), _stream()), "bn_batch_moments")
    return moments


def bn_relu_fwd_from_moments(d, x, gamma, beta, residual, y, moments, save_mean, save_invstd):
    _check(lib().bn_relu_fwd_from_moments(ctypes.byref(d), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(residual), _ptr(y),
                                          _ptr(moments), _ptr(save_mean), _ptr(save_invstd), _stream()), "bn_relu_fwd_from_moments")
    return y


def bn_relu_bwd_sums(d, dy, x, y, save_mean, save_invstd, sums, ws=None):
    ws = ws if ws is not None else _ws(bn_workspace_bytes(d), x)
    _check(lib().bn_relu_bwd_sums(ctypes.byref(d), _ptr(dy), _ptr(x), _ptr(y), _ptr(save_mean), _ptr(save_invstd), _ptr(sums),
                                  _ptr(ws), ws.numel(), _stream()), "bn_relu_bwd_sums")
    return sums


def bn_relu_bwd_from_sums(d, dy, x, y, gamma, save_mean, save_invstd, sums, total_rows, dx, dresidual):
    _check(lib().bn_relu_bwd_from_sums(ctypes.byref(d), _ptr(dy), _ptr(x), _ptr(y), _ptr(gamma), _ptr(save_mean),
                                       _ptr(save_invstd), _ptr(sums), int(total_rows), _ptr(dx), _ptr(dresidual), _stream()),
           "bn_relu_bwd_from_sums")
    return dx


def ls_xent_fwd_bwd(batch, classes, logits, labels, eps, grad_scale, loss_mean, loss_per_sample, dlogits,
                    dlogits_dt=RN50_F16):
    _check(lib().ls_xent_fwd_bwd(batch, classes, _ptr(logits), _ptr(labels), eps, grad_scale, _ptr(loss_mean),
                                 _ptr(loss_per_sample), _ptr(dlogits), dlogits_dt, _stream()), "ls_xent_fwd_bwd")


def sgd_momentum_flat(n, grad, grad_scale, master_w, momentum, w_lowp_out, lr, mu, wd, grad_dt=RN50_F16):
    _check(lib().sgd_momentum_flat(n, _ptr(grad), grad_dt, grad_scale, _ptr(master_w), _ptr(momentum),
                                   _ptr(w_lowp_out), lr, mu, wd, _stream()), "sgd_momentum_flat")


def sched_lr_b(epoch):
    return float(lib().rn50_sched_lr_b(float(epoch)))


def sched_momentum_b(epoch, total_batch):
    return float(lib().rn50_sched_momentum_b(float(epoch), float(total_batch)))


def sched_batch(experiment, epoch):
    """(per-worker, total) mini-batch size of Table 3's experiment at `epoch`."""
    pw, tot = _i(), _i()
    _check(lib().rn50_sched_batch(experiment, float(epoch), ctypes.byref(pw), ctypes.byref(tot)), "rn50_sched_batch")
    return pw.value, tot.value


class LarsPlan:
    """Device tables for lars_momentum_flat over segments [(offset, count, use_lars), ...]; owns its workspace."""

    def __init__(self, segments, device):
        import torch
        self.nseg = len(segments)
        arr = (rn50_lars_segment * max(self.nseg, 1))(*[rn50_lars_segment(int(o), int(c), 1 if u else 0) for o, c, u in segments])
        need = int(lib().lars_workspace_bytes(arr, self.nseg))
        if need == 0 and self.nseg:
            raise Rn50Error("lars_workspace_bytes: bad segment table")
        self.workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=device)
        h = _vp()
        _check(lib().lars_plan_create(ctypes.byref(h), arr, self.nseg, _ptr(self.workspace), need), "lars_plan_create")
        self.handle = h

    def step(self, grad, grad_scale, master_w, momentum, w_lowp_out, lr, mu, wd, eta, eps, rates_out=None, grad_dt=RN50_F16):
        _check(lib().lars_momentum_flat(self.handle, _ptr(grad), grad_dt, grad_scale, _ptr(master_w), _ptr(momentum),
                                        _ptr(w_lowp_out), lr, mu, wd, eta, eps, _ptr(rates_out), _stream()), "lars_momentum_flat")

    def close(self):
        if self.handle:
            lib().lars_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def rn50_cast_params(n, master_w, w_lowp, dt=RN50_F16):
    _check(lib().rn50_cast_params(n, _ptr(master_w), _ptr(w_lowp), dt, _stream()), "rn50_cast_params")


def rn50_profile_begin():
    _check(lib().rn50_profile_begin(), "rn50_profile_begin")


def rn50_profile_end():
    """List of dicts (name, launches, total_ms, flops, bytes, side_launches), one per kernel that ran."""
    buf = (rn50_profile_entry * 64)()
    n = _i()
    _check(lib().rn50_profile_end(buf, 64, ctypes.byref(n)), "rn50_profile_end")
    return [dict(name=buf[i].name.decode(), launches=int(buf[i].launches), total_ms=float(buf[i].total_ms),
                 flops=float(buf[i].flops), bytes=float(buf[i].bytes), side_launches=int(buf[i].side_launches))
            for i in range(n.value)]


# ------------------------------------------------------------------ whole step
def make_config(batch, image_hw=(224, 224), has_stem=True, blocks=(3, 4, 6, 3), base_width=64, classes=1000,
                bn_eps=1e-5, ls_eps=0.1, loss_scale=1.0, dt=RN50_F16, keep_grads=False):
    b = (ctypes.c_int * 4)(*(list(blocks) + [0] * (4 - len(blocks))))
    return rn50_config(batch, image_hw[0], image_hw[1], int(has_stem), len(blocks), b, base_width, classes, dt,
                       bn_eps, ls_eps, loss_scale, int(keep_grads))


def rn50_param_count(cfg):
    return int(lib().rn50_param_count(ctypes.byref(cfg)))


def rn50_param_layout(cfg):
    """List of (kind, offset, count, fan_in) for every segment of the flat layout."""
    l = lib()
    out = []
    for i in range(l.rn50_num_segments(ctypes.byref(cfg))):
        off, cnt, kind, fan = _sz(), _sz(), _i(), _i()
        _check(l.rn50_param_layout(ctypes.byref(cfg), i, ctypes.byref(off), ctypes.byref(cnt), ctypes.byref(kind),
                                   ctypes.byref(fan)), "rn50_param_layout")
        out.append((kind.value, off.value, cnt.value, fan.value))
    return out


def rn50_workspace_bytes(cfg):
    return int(lib().rn50_workspace_bytes(ctypes.byref(cfg)))


def probe_mfma(blocks, iters, out):
    """Register-only MFMA loop (rn50_probe_mfma); out: float tensor of blocks*256 elements."""
    _check(lib().rn50_probe_mfma(int(blocks), int(iters), _ptr(out), _stream()), "rn50_probe_mfma")


def probe_tile_load(src, src_bytes, blocks, iters, start_stride, through_lds, out):
    _check(lib().rn50_probe_tile_load(_ptr(src), int(src_bytes), int(blocks), int(iters), int(start_stride),
                                      int(bool(through_lds)), _ptr(out), _stream()), "rn50_probe_tile_load")


def probe_copy(src, dst, nbytes):
    _check(lib().rn50_probe_copy(_ptr(src), _ptr(dst), int(nbytes), _stream()), "rn50_probe_copy")


def probe_empty(count=1):
    _check(lib().rn50_probe_empty(int(count), _stream()), "rn50_probe_empty")


def conv_variant_applies(d, which, variant):
    """True if the variant id names a kernel of its own for this shape (no GPU needed)."""
    return bool(lib().rn50_conv_variant_applies(ctypes.byref(d), int(which), int(variant)))


def shipped_tuning_path(batch):
    """File of the kernel-variant table shipped for full ResNet-50 at this per-GPU batch size (written by
    tune_in_situ on an MI355X), or None if none is shipped for it."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tuning_resnet50_b%d.json" % int(batch))
    return path if os.path.exists(path) else None


def shipped_tuning(batch):
    """The shipped variant table ([fwd, dgrad, wgrad] per convolution, for Rn50Context.set_tuning) or None."""
    path = shipped_tuning_path(batch)
    if path is None:
        return None
    import json
    with open(path) as f:
        return json.load(f)["table"]


class Rn50Context:
    """Owns the workspace tensor and the rn50_ctx handle."""

    def __init__(self, cfg, device="cuda:0"):
        import torch
        self.cfg = cfg
        nbytes = rn50_workspace_bytes(cfg)
        if nbytes == 0:
            raise Rn50Error("rn50_workspace_bytes: bad configuration")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        h = _vp()
        _check(lib().rn50_create(ctypes.byref(h), ctypes.byref(cfg), _ptr(self.workspace), nbytes), "rn50_create")
        self.handle = h

    def step(self, images, labels, master_w, momentum, w_lowp, grad_lowp, hp, loss_out):
        hpp = None if hp is None else ctypes.byref(hp)
        _check(lib().rn50_step(self.handle, _ptr(images), _ptr(labels), _ptr(master_w), _ptr(momentum),
                               _ptr(w_lowp), _ptr(grad_lowp), hpp, _ptr(loss_out), _stream()), "rn50_step")

    def autotune(self, images, labels, master_w, w_lowp, grad_lowp, loss_out):
        """Time the kernel variants of every convolution on one forward+backward pass (synchronises)."""
        _check(lib().rn50_autotune(self.handle, _ptr(images), _ptr(labels), _ptr(master_w), _ptr(w_lowp),
                                   _ptr(grad_lowp), _ptr(loss_out), _stream()), "rn50_autotune")

    def get_tuning(self):
        """Kernel variants in use: [fwd, dgrad, wgrad] per convolution in network order (-1 = heuristic)."""
        n = lib().rn50_get_tuning(self.handle, None, 0)
        buf = (_i * n)()
        if lib().rn50_get_tuning(self.handle, buf, n) != n:
            raise Rn50Error("rn50_get_tuning failed")
        return list(buf)

    def set_tuning(self, table):
        buf = (_i * len(table))(*[int(v) for v in table])
        _check(lib().rn50_set_tuning(self.handle, buf, len(table)), "rn50_set_tuning")

    def tuning_report(self):
        n = int(lib().rn50_tuning_report(self.handle, None, 0))
        buf = ctypes.create_string_buffer(n + 1)
        lib().rn50_tuning_report(self.handle, buf, n + 1)
        return buf.value.decode()

    def tensor(self, name):
        """Copy of a workspace tensor left by the last step, as a flat torch tensor (half or float)."""
        import torch
        p, n, eb = _vp(), _sz(), _i()
        _check(lib().rn50_tensor(self.handle, name.encode(), ctypes.byref(p), ctypes.byref(n), ctypes.byref(eb)),
               "rn50_tensor(%s)" % name)
        base = self.workspace.data_ptr()
        off = p.value - base
        raw = self.workspace[off:off + n.value * eb.value]
        return raw.view(torch.float16 if eb.value == 2 else torch.float32).clone()

    def close(self):
        if self.handle:
            lib().rn50_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
