"""ctypes binding of libsp3d.so: same names as the C ABI (include/sp3d.h), argument
marshalling only.  Tensors are torch tensors on the GPU (used for their device memory and
stream); every operation runs in the library's HIP kernels.  There is no CPU fallback: if the
library has not been built the import of the library raises.
"""
import ctypes
import os

SP_F32, SP_BF16 = 0, 1
SP_OK, SP_EINVAL, SP_EGEOM, SP_EUNSUPPORTED, SP_EWORKSPACE, SP_ELAUNCH = 0, -1, -2, -3, -4, -5
SP_FLAG_RELU = 1
SP_HALO_SKIP_SEND, SP_HALO_KEEP_ZERO, SP_HALO_GATHER = 1, 2, 4
SP_STATIC_SCRATCH_BYTES = 32 << 20
SP_OP_FWD, SP_OP_DGRAD, SP_OP_WGRAD, SP_OP_UPCONV_WGRAD, SP_OP_POINTWISE_WGRAD, SP_OP_LOSS = 0, 1, 2, 3, 4, 5

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsp3d.so")

EXPORTS = ["sp_padded_elems", "sp_msg_elems", "sp_workspace_bytes", "sp_check_geom", "sp_gather_supported", "sp_strerror",
           "sp_last_hip_error", "sp_partition", "sp_unpartition", "halo_pack", "halo_unpack",
           "sp_halo_exchange",
           "conv3d_fwd", "conv3d_dgrad", "conv3d_dgrad_relu", "sp_relu_bits_bytes", "sp_relu_bits_supported", "sp_relu_bits",
           "conv3d_fwd_bits", "conv3d_fwd2_bits", "conv3d_dgrad_bits", "conv3d_wgrad", "conv3d_wgrad_static", "conv3d_fwd2", "conv3d_dgrad2",
           "conv3d_wgrad2", "sp_relu_bwd",
           "sp_maxpool2_fwd", "sp_maxpool2_bwd", "sp_maxpool2_bwd_join", "sp_upconv2_fwd", "sp_upconv2_dgrad", "sp_upconv2_wgrad",
           "sp_pointwise_fwd", "sp_pointwise_dgrad", "sp_pointwise_dgrad_relu", "sp_pointwise_wgrad", "sp_pointwise_bwd_relu", "sp_concat", "sp_split", "sp_add",
           "sp_dice_ce_loss"]


class Geom(ctypes.Structure):
    """sp_geom_t: volume extents, tile grid (D,H,W order), margin width of the layout, and by how much the
    convolutions grow their output box beyond the interior (0 unless several layers share one exchange).
    flat = 1 selects the 2-D variant: D is a stack of independent slices (3x3 kernels, 1x2x2 windows)."""
    _fields_ = [(k, ctypes.c_int32) for k in ("n", "d", "h", "w", "gd", "gh", "gw", "halo", "grow", "flat", "opts")]

    def __init__(self, n, dhw, grid, halo=1, grow=0, flat=0, opts=0):
        super().__init__(n, dhw[0], dhw[1], dhw[2], grid[0], grid[1], grid[2], halo, grow, int(flat), opts)

    def grown(self, grow):
        """The same geometry with another `grow`."""
        return Geom(self.n, (self.d, self.h, self.w), (self.gd, self.gh, self.gw), self.halo, grow, self.flat,
                    self.opts)

    def with_opts(self, opts):
        """The same geometry with other SP_HALO_* flags."""
        return Geom(self.n, (self.d, self.h, self.w), (self.gd, self.gh, self.gw), self.halo, self.grow, self.flat,
                    opts)

    @property
    def tile(self):
        return self.d // self.gd, self.h // self.gh, self.w // self.gw

    @property
    def padded_shape(self):
        """Shape of the padded tile array without the channel axis."""
        t = self.tile
        return (self.n, self.gd, self.gh, self.gw) + tuple(e + 2 * self.halo for e in t)


class Sp3dError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (code %d, hip error %d)" % (
            where, lib().sp_strerror(code).decode(), code, lib().sp_last_hip_error()))


_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libsp3d.so is not built: run `python -c 'import __graft_entry__ as g;"
                              " g.build()'` (or paper_1909_03108_amd/build.py) first")
        L = ctypes.CDLL(LIB_PATH)
        G, P, I, U, Z = ctypes.POINTER(Geom), ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32, ctypes.c_size_t
        L.sp_padded_elems.argtypes, L.sp_padded_elems.restype = [G, I], Z
        L.sp_msg_elems.argtypes, L.sp_msg_elems.restype = [G, I], Z
        L.sp_workspace_bytes.argtypes, L.sp_workspace_bytes.restype = [I, G, I, I, I], Z
        L.sp_check_geom.argtypes, L.sp_check_geom.restype = [G], I
        L.sp_gather_supported.argtypes, L.sp_gather_supported.restype = [I, G, I, I, I], I
        L.sp_strerror.argtypes, L.sp_strerror.restype = [I], ctypes.c_char_p
        L.sp_last_hip_error.argtypes, L.sp_last_hip_error.restype = [], I
        for name in ("sp_partition", "sp_unpartition", "halo_pack", "halo_unpack"):
            f = getattr(L, name)
            f.argtypes, f.restype = [P, P, G, I, I, P], I
        L.sp_halo_exchange.argtypes, L.sp_halo_exchange.restype = [P, G, I, I, P], I
        L.conv3d_fwd.argtypes, L.conv3d_fwd.restype = [P, P, P, P, G, I, I, I, U, P, Z, P], I
        L.conv3d_dgrad.argtypes, L.conv3d_dgrad.restype = [P, P, P, G, I, I, I, P, Z, P], I
        L.conv3d_dgrad_relu.argtypes, L.conv3d_dgrad_relu.restype = [P, P, P, P, G, I, I, I, P, Z, P], I
        L.sp_relu_bits_bytes.argtypes, L.sp_relu_bits_bytes.restype = [G, I], Z
        L.sp_relu_bits_supported.argtypes, L.sp_relu_bits_supported.restype = [I, G, I, I, I], I
        L.sp_relu_bits.argtypes, L.sp_relu_bits.restype = [P, P, G, I, I, P], I
        L.conv3d_fwd_bits.argtypes, L.conv3d_fwd_bits.restype = [P, P, P, P, P, G, I, I, I, U, P, Z, P], I
        L.conv3d_fwd2_bits.argtypes, L.conv3d_fwd2_bits.restype = [P, I, P, I, P, P, P, P, G, I, I, U, P, Z, P], I
        L.conv3d_dgrad_bits.argtypes, L.conv3d_dgrad_bits.restype = [P, P, P, P, G, I, I, I, P, Z, P], I
        L.conv3d_wgrad.argtypes, L.conv3d_wgrad.restype = [P, P, P, P, G, I, I, I, P, Z, P], I
        L.conv3d_wgrad_static.argtypes, L.conv3d_wgrad_static.restype = [P, P, P, P, G, I, I, I, P], I
        L.conv3d_fwd2.argtypes, L.conv3d_fwd2.restype = [P, I, P, I, P, P, P, G, I, I, U, P, Z, P], I
        L.conv3d_dgrad2.argtypes, L.conv3d_dgrad2.restype = [P, P, P, I, P, I, G, I, I, P, Z, P], I
        L.conv3d_wgrad2.argtypes, L.conv3d_wgrad2.restype = [P, I, P, I, P, P, P, G, I, I, P, Z, P], I
        L.sp_relu_bwd.argtypes, L.sp_relu_bwd.restype = [P, P, P, G, I, I, P], I
        L.sp_maxpool2_fwd.argtypes, L.sp_maxpool2_fwd.restype = [P, P, G, I, I, P], I
        L.sp_maxpool2_bwd.argtypes, L.sp_maxpool2_bwd.restype = [P, P, P, G, I, I, P], I
        L.sp_maxpool2_bwd_join.argtypes, L.sp_maxpool2_bwd_join.restype = [P, P, P, P, G, I, I, P], I
        L.sp_upconv2_fwd.argtypes, L.sp_upconv2_fwd.restype = [P, P, P, P, G, I, I, I, P], I
        L.sp_upconv2_dgrad.argtypes, L.sp_upconv2_dgrad.restype = [P, P, P, G, I, I, I, P], I
        L.sp_upconv2_wgrad.argtypes, L.sp_upconv2_wgrad.restype = [P, P, P, P, G, I, I, I, P, Z, P], I
        L.sp_pointwise_fwd.argtypes, L.sp_pointwise_fwd.restype = [P, P, P, P, G, I, I, I, U, P], I
        L.sp_pointwise_dgrad.argtypes, L.sp_pointwise_dgrad.restype = [P, P, P, G, I, I, I, P], I
        L.sp_pointwise_dgrad_relu.argtypes, L.sp_pointwise_dgrad_relu.restype = [P, P, P, P, G, I, I, I, P], I
        L.sp_pointwise_wgrad.argtypes, L.sp_pointwise_wgrad.restype = [P, P, P, P, G, I, I, I, P, Z, P], I
        L.sp_pointwise_bwd_relu.argtypes, L.sp_pointwise_bwd_relu.restype = [P, P, P, P, P, P, G, I, I, I, P, Z, P], I
        L.sp_concat.argtypes, L.sp_concat.restype = [P, I, P, I, P, G, I, P], I
        L.sp_split.argtypes, L.sp_split.restype = [P, P, I, P, I, G, I, P], I
        L.sp_add.argtypes, L.sp_add.restype = [P, P, P, G, I, I, P], I
        F = ctypes.c_float
        L.sp_dice_ce_loss.argtypes, L.sp_dice_ce_loss.restype = [P, P, P, P, P, G, I, I, F, F, F, P, Z, P], I
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _check(rc, where):
    if rc != SP_OK:
        raise Sp3dError(rc, where)


def sp_padded_elems(g, c):
    return lib().sp_padded_elems(ctypes.byref(g), c)


def sp_msg_elems(g, c):
    return lib().sp_msg_elems(ctypes.byref(g), c)


def sp_gather_supported(op, g, cin, cout, dt):
    return bool(lib().sp_gather_supported(op, ctypes.byref(g), cin, cout, dt))


def sp_workspace_bytes(op, g, cin, cout, dt):
    r = lib().sp_workspace_bytes(op, ctypes.byref(g), cin, cout, dt)
    if r == ctypes.c_size_t(-1).value:
        raise Sp3dError(SP_EUNSUPPORTED, "sp_workspace_bytes")
    return r


def sp_check_geom(g):
    return lib().sp_check_geom(ctypes.byref(g))


def sp_partition(vol, P, g, c, dt, stream=None):
    _check(lib().sp_partition(_ptr(vol), _ptr(P), ctypes.byref(g), c, dt, _stream(stream)), "sp_partition")


def sp_unpartition(P, vol, g, c, dt, stream=None):
    _check(lib().sp_unpartition(_ptr(P), _ptr(vol), ctypes.byref(g), c, dt, _stream(stream)),
           "sp_unpartition")


def halo_pack(P, msg, g, c, dt, stream=None):
    _check(lib().halo_pack(_ptr(P), _ptr(msg), ctypes.byref(g), c, dt, _stream(stream)), "halo_pack")


def halo_unpack(P, msg, g, c, dt, stream=None):
    _check(lib().halo_unpack(_ptr(P), _ptr(msg), ctypes.byref(g), c, dt, _stream(stream)), "halo_unpack")


def sp_halo_exchange(P, g, c, dt, stream=None):
    _check(lib().sp_halo_exchange(_ptr(P), ctypes.byref(g), c, dt, _stream(stream)), "sp_halo_exchange")


def conv3d_fwd(Px, w, bias, Py, g, cin, cout, dt, flags=0, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_fwd(_ptr(Px), _ptr(w), _ptr(bias), _ptr(Py), ctypes.byref(g), cin, cout, dt,
                            flags, wp, wb, _stream(stream)), "conv3d_fwd")


def conv3d_dgrad(Pdz, w, Pdx, g, cin, cout, dt, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_dgrad(_ptr(Pdz), _ptr(w), _ptr(Pdx), ctypes.byref(g), cin, cout, dt, wp, wb,
                              _stream(stream)), "conv3d_dgrad")


def conv3d_dgrad_relu(Pdz, w, Px, Pdx, g, cin, cout, dt, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_dgrad_relu(_ptr(Pdz), _ptr(w), _ptr(Px), _ptr(Pdx), ctypes.byref(g), cin, cout, dt, wp, wb,
                                   _stream(stream)), "conv3d_dgrad_relu")


def sp_relu_bits_bytes(g, c):
    return lib().sp_relu_bits_bytes(ctypes.byref(g), c)


def sp_relu_bits_supported(op, g, cin, cout, dt):
    return bool(lib().sp_relu_bits_supported(op, ctypes.byref(g), cin, cout, dt))


def sp_relu_bits(Py, bits, g, c, dt, stream=None):
    _check(lib().sp_relu_bits(_ptr(Py), _ptr(bits), ctypes.byref(g), c, dt, _stream(stream)), "sp_relu_bits")


def conv3d_fwd_bits(Px, w, bias, Py, bits, g, cin, cout, dt, flags=0, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_fwd_bits(_ptr(Px), _ptr(w), _ptr(bias), _ptr(Py), _ptr(bits), ctypes.byref(g), cin, cout, dt,
                                 flags, wp, wb, _stream(stream)), "conv3d_fwd_bits")


def conv3d_fwd2_bits(Pxa, ca, Pxb, cb, w, bias, Py, bits, g, cout, dt, flags=0, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_fwd2_bits(_ptr(Pxa), ca, _ptr(Pxb), cb, _ptr(w), _ptr(bias), _ptr(Py), _ptr(bits),
                                  ctypes.byref(g), cout, dt, flags, wp, wb, _stream(stream)), "conv3d_fwd2_bits")


def conv3d_dgrad_bits(Pdz, w, bits, Pdx, g, cin, cout, dt, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_dgrad_bits(_ptr(Pdz), _ptr(w), _ptr(bits), _ptr(Pdx), ctypes.byref(g), cin, cout, dt, wp, wb,
                                   _stream(stream)), "conv3d_dgrad_bits")


def conv3d_fwd2(Pxa, ca, Pxb, cb, w, bias, Py, g, cout, dt, flags=0, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_fwd2(_ptr(Pxa), ca, _ptr(Pxb), cb, _ptr(w), _ptr(bias), _ptr(Py), ctypes.byref(g), cout, dt,
                             flags, wp, wb, _stream(stream)), "conv3d_fwd2")


def conv3d_dgrad2(Pdz, w, Pdxa, ca, Pdxb, cb, g, cout, dt, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_dgrad2(_ptr(Pdz), _ptr(w), _ptr(Pdxa), ca, _ptr(Pdxb), cb, ctypes.byref(g), cout, dt, wp, wb,
                               _stream(stream)), "conv3d_dgrad2")


def conv3d_wgrad2(Pxa, ca, Pxb, cb, Pdz, dw, db, g, cout, dt, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_wgrad2(_ptr(Pxa), ca, _ptr(Pxb), cb, _ptr(Pdz), _ptr(dw), _ptr(db), ctypes.byref(g), cout, dt,
                               wp, wb, _stream(stream)), "conv3d_wgrad2")


def conv3d_wgrad(Px, Pdz, dw, db, g, cin, cout, dt, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().conv3d_wgrad(_ptr(Px), _ptr(Pdz), _ptr(dw), _ptr(db), ctypes.byref(g), cin, cout, dt,
                              wp, wb, _stream(stream)), "conv3d_wgrad")


def conv3d_wgrad_static(Px, Pdz, dw, db, g, cin, cout, dt, stream=None):
    _check(lib().conv3d_wgrad_static(_ptr(Px), _ptr(Pdz), _ptr(dw), _ptr(db), ctypes.byref(g), cin, cout, dt,
                                     _stream(stream)), "conv3d_wgrad_static")


def sp_relu_bwd(Pdy, Py, Pdz, g, c, dt, stream=None):
    _check(lib().sp_relu_bwd(_ptr(Pdy), _ptr(Py), _ptr(Pdz), ctypes.byref(g), c, dt, _stream(stream)),
           "sp_relu_bwd")


def sp_maxpool2_fwd(Px, Py, gf, c, dt, stream=None):
    _check(lib().sp_maxpool2_fwd(_ptr(Px), _ptr(Py), ctypes.byref(gf), c, dt, _stream(stream)), "sp_maxpool2_fwd")


def sp_maxpool2_bwd(Px, Pdy, Pdx, gf, c, dt, stream=None):
    _check(lib().sp_maxpool2_bwd(_ptr(Px), _ptr(Pdy), _ptr(Pdx), ctypes.byref(gf), c, dt, _stream(stream)),
           "sp_maxpool2_bwd")


def sp_maxpool2_bwd_join(Px, Pdy, Pskip, Pdz, gf, c, dt, stream=None):
    _check(lib().sp_maxpool2_bwd_join(_ptr(Px), _ptr(Pdy), _ptr(Pskip), _ptr(Pdz), ctypes.byref(gf), c, dt,
                                      _stream(stream)), "sp_maxpool2_bwd_join")


def sp_upconv2_fwd(Px, u, bias, Py, gf, cin, cout, dt, stream=None):
    _check(lib().sp_upconv2_fwd(_ptr(Px), _ptr(u), _ptr(bias), _ptr(Py), ctypes.byref(gf), cin, cout, dt,
                                _stream(stream)), "sp_upconv2_fwd")


def sp_upconv2_dgrad(Pdy, u, Pdx, gf, cin, cout, dt, stream=None):
    _check(lib().sp_upconv2_dgrad(_ptr(Pdy), _ptr(u), _ptr(Pdx), ctypes.byref(gf), cin, cout, dt,
                                  _stream(stream)), "sp_upconv2_dgrad")


def sp_upconv2_wgrad(Px, Pdy, du, db, gf, cin, cout, dt, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().sp_upconv2_wgrad(_ptr(Px), _ptr(Pdy), _ptr(du), _ptr(db), ctypes.byref(gf), cin, cout, dt,
                                  wp, wb, _stream(stream)), "sp_upconv2_wgrad")


def sp_pointwise_fwd(Px, p, bias, Py, g, cin, cout, dt, flags=0, stream=None):
    _check(lib().sp_pointwise_fwd(_ptr(Px), _ptr(p), _ptr(bias), _ptr(Py), ctypes.byref(g), cin, cout, dt,
                                  flags, _stream(stream)), "sp_pointwise_fwd")


def sp_pointwise_dgrad(Pdy, p, Pdx, g, cin, cout, dt, stream=None):
    _check(lib().sp_pointwise_dgrad(_ptr(Pdy), _ptr(p), _ptr(Pdx), ctypes.byref(g), cin, cout, dt,
                                    _stream(stream)), "sp_pointwise_dgrad")


def sp_pointwise_dgrad_relu(Pdy, p, Px, Pdx, g, cin, cout, dt, stream=None):
    _check(lib().sp_pointwise_dgrad_relu(_ptr(Pdy), _ptr(p), _ptr(Px), _ptr(Pdx), ctypes.byref(g), cin, cout, dt,
                                         _stream(stream)), "sp_pointwise_dgrad_relu")


def sp_pointwise_bwd_relu(Px, Pdy, p, Pdx, dp, db, g, cin, cout, dt, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().sp_pointwise_bwd_relu(_ptr(Px), _ptr(Pdy), _ptr(p), _ptr(Pdx), _ptr(dp), _ptr(db), ctypes.byref(g),
                                       cin, cout, dt, wp, wb, _stream(stream)), "sp_pointwise_bwd_relu")


def sp_pointwise_wgrad(Px, Pdy, dp, db, g, cin, cout, dt, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().sp_pointwise_wgrad(_ptr(Px), _ptr(Pdy), _ptr(dp), _ptr(db), ctypes.byref(g), cin, cout, dt,
                                    wp, wb, _stream(stream)), "sp_pointwise_wgrad")


def sp_concat(Pa, ca, Pb, cb, Pout, g, dt, stream=None):
    _check(lib().sp_concat(_ptr(Pa), ca, _ptr(Pb), cb, _ptr(Pout), ctypes.byref(g), dt, _stream(stream)),
           "sp_concat")


def sp_split(Pin, Pa, ca, Pb, cb, g, dt, stream=None):
    _check(lib().sp_split(_ptr(Pin), _ptr(Pa), ca, _ptr(Pb), cb, ctypes.byref(g), dt, _stream(stream)),
           "sp_split")


def sp_add(Pa, Pb, Pout, g, c, dt, stream=None):
    _check(lib().sp_add(_ptr(Pa), _ptr(Pb), _ptr(Pout), ctypes.byref(g), c, dt, _stream(stream)), "sp_add")


def coarse_geom(gf):
    """Geometry of the half-resolution side of a pooling / up-convolution on the same tile grid (the 2-D
    variant keeps D: its windows are 1x2x2)."""
    return Geom(gf.n, (gf.d if gf.flat else gf.d // 2, gf.h // 2, gf.w // 2), (gf.gd, gf.gh, gf.gw), gf.halo, 0,
                gf.flat)


# ---- plumbing helpers (device memory only; no arithmetic) ---------------------------------------

def torch_dtype(dt):
    import torch
    return torch.bfloat16 if dt == SP_BF16 else torch.float32


def alloc_padded(g, c, dt, zero=True, device="cuda"):
    """Device buffer for the padded tile array P[n,gd,gh,gw,pd,ph,pw,c]."""
    import torch
    f = torch.zeros if zero else torch.empty
    return f(g.padded_shape + (c,), dtype=torch_dtype(dt), device=device)


def alloc_msg(g, c, dt, device="cuda"):
    import torch
    return torch.empty((sp_msg_elems(g, c),), dtype=torch_dtype(dt), device=device)


def alloc_ws(nbytes, device="cuda"):
    import torch
    return torch.empty((max(int(nbytes), 16),), dtype=torch.uint8, device=device)


def sp_dice_ce_loss(Plogits, Plabels, Pdlogits, loss, stats, g, classes, dt, w_dice=0.9, w_ce=0.1, eps=1.0, ws=None,
                    stream=None):
    wp, wb = _ws(ws)
    _check(lib().sp_dice_ce_loss(_ptr(Plogits), _ptr(Plabels), _ptr(Pdlogits), _ptr(loss), _ptr(stats),
                                 ctypes.byref(g), classes, dt, w_dice, w_ce, eps, wp, wb, _stream(stream)),
           "sp_dice_ce_loss")
