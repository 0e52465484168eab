// C-ABI entry points of libsp3d: argument checks, workspace sizing, kernel dispatch.
// Every check happens on the host before anything is enqueued.
#include "common.h"

#include <atomic>
#include <mutex>

namespace sp3d {

static std::atomic<int> g_last_hip_error{0};

// Scratch memory of conv3d_wgrad_static: one copy per GPU, held from module load until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; every use of the memory (kernel
// arguments) goes through the per-device address that static_scratch() returns.
static __device__ __align__(256) unsigned char scratch[SP_STATIC_SCRATCH_BYTES];

static int static_scratch(void **out) {
    enum { kMaxDevices = 64 };
    static std::mutex mu;
    static void *addr[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return record_hip(e);
    if (dev < 0 || dev >= kMaxDevices) return SP_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {            // first call on this device, with it current: look its copy up once
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return record_hip(e);
        if (!p) return SP_ELAUNCH;
        addr[dev] = p;
    }
    *out = addr[dev];
    return SP_OK;
}

int record_hip(hipError_t e) {
    if (e == hipSuccess) return SP_OK;
    g_last_hip_error.store(static_cast<int>(e));
    return SP_ELAUNCH;
}

int make_geo(const sp_geom_t *g, Geo *out) {
    if (!g) return SP_EINVAL;
    if (g->n <= 0 || g->d <= 0 || g->h <= 0 || g->w <= 0 || g->gd <= 0 || g->gh <= 0 ||
        g->gw <= 0 || g->halo < 0 || g->grow < 0 || (g->grow > 0 && g->grow >= g->halo) ||
        (g->flat != 0 && g->flat != 1) || (g->opts & ~(SP_HALO_SKIP_SEND | SP_HALO_KEEP_ZERO | SP_HALO_GATHER)))
        return SP_EINVAL;
    if (g->d % g->gd || g->h % g->gh || g->w % g->gw) return SP_EGEOM;
    if (g->halo < 1 || g->halo > SP_MAX_HALO) return SP_EUNSUPPORTED;
    Geo o;
    o.n = g->n; o.gd = g->gd; o.gh = g->gh; o.gw = g->gw;
    o.td = g->d / g->gd; o.th = g->h / g->gh; o.tw = g->w / g->gw;
    o.halo = g->halo;
    o.grow = g->grow;
    o.flat = g->flat;
    // (the 2-D variant moves nothing along D, so a tile may hold fewer slices than the margin is wide)
    if ((!o.flat && o.td < o.halo) || o.th < o.halo || o.tw < o.halo) return SP_EGEOM;
    o.pd = o.td + 2 * o.halo; o.ph = o.th + 2 * o.halo; o.pw = o.tw + 2 * o.halo;
    long long nt = 1LL * o.n * o.gd * o.gh * o.gw;
    if (nt > 0x7fffffffLL) return SP_EGEOM;
    o.ntiles = static_cast<int>(nt);
    o.tile_vox = 1LL * o.pd * o.ph * o.pw;
    o.int_vox = 1LL * o.td * o.th * o.tw;
    o.msg_vox = o.tile_vox - o.int_vox;
    if (o.tile_vox > 0x7fffffffLL) return SP_EGEOM;   // per-tile voxel indices stay 32-bit
    if (out) *out = o;
    return SP_OK;
}

void make_regions(const Geo &g, RegionTable *t) {
    const int ext[3] = {g.td, g.th, g.tw};
    int k = 0;
    long long off = 0;
    for (int dd = -1; dd <= 1; ++dd)
        for (int dh = -1; dh <= 1; ++dh)
            for (int dw = -1; dw <= 1; ++dw) {
                if (!dd && !dh && !dw) continue;
                Region &r = t->r[k];
                const int dl[3] = {dd, dh, dw};
                long long n = 1;
                for (int a = 0; a < 3; ++a) {
                    r.delta[a] = dl[a];
                    r.ext[a] = dl[a] ? g.halo : ext[a];
                    // sent box: own voxels nearest to the neighbour (padded coordinates)
                    r.send[a] = g.halo + (dl[a] > 0 ? ext[a] - g.halo : 0);
                    // margin box lying in direction delta
                    r.recv[a] = dl[a] < 0 ? 0 : (dl[a] == 0 ? g.halo : g.halo + ext[a]);
                    n *= r.ext[a];
                }
                r.off = off;
                off += n;
                r.opposite = 25 - k;   // lexicographic order is symmetric under negation
                ++k;
            }
}

static bool chan_ok(int c) { return c > 0 && c <= 4096; }
static bool dtype_ok(sp_dtype_t dt) { return dt == SP_F32 || dt == SP_BF16; }

static bool overlap(const void *a, size_t na, const void *b, size_t nb) {
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + nb && y < x + na;
}

}  // namespace sp3d

using namespace sp3d;

extern "C" {

size_t sp_padded_elems(const sp_geom_t *g, int c) {
    Geo o;
    if (make_geo(g, &o) != SP_OK || c <= 0) return 0;
    return static_cast<size_t>(o.ntiles) * o.tile_vox * c;
}

size_t sp_msg_elems(const sp_geom_t *g, int c) {
    Geo o;
    if (make_geo(g, &o) != SP_OK || c <= 0) return 0;
    return static_cast<size_t>(o.ntiles) * o.msg_vox * c;
}

int sp_check_geom(const sp_geom_t *g) { return make_geo(g, nullptr); }

int sp_gather_supported(int op, const sp_geom_t *g, int cin, int cout, sp_dtype_t dt) {
    Geo o;
    if (make_geo(g, &o) != SP_OK || !chan_ok(cin) || !chan_ok(cout) || !dtype_ok(dt)) return 0;
    switch (op) {
    case SP_OP_FWD: return conv_mfma_gather_supported(o, cin, cout, dt) ? 1 : 0;
    case SP_OP_DGRAD: return conv_mfma_gather_supported(o, cout, cin, dt) ? 1 : 0;     // channel roles swapped
    case SP_OP_WGRAD: return wgrad_mfma_gather_supported(o, cin, cout, dt) ? 1 : 0;
    default: return 0;
    }
}

size_t sp_workspace_bytes(int op, const sp_geom_t *g, int cin, int cout, sp_dtype_t dt) {
    Geo o;
    if (make_geo(g, &o) != SP_OK || !chan_ok(cin) || !chan_ok(cout) || !dtype_ok(dt))
        return static_cast<size_t>(-1);
    switch (op) {
    case SP_OP_FWD:
    case SP_OP_DGRAD: {
        // dgrad swaps the channel roles of the same kernel
        const int ki = op == SP_OP_FWD ? cin : cout, ko = op == SP_OP_FWD ? cout : cin;
        if (conv_mfma_supported(o, ki, ko, dt)) return conv_mfma_ws_bytes(o, ki, ko);
        if (op == SP_OP_FWD && !conv_c1_supported(o, cin, cout, dt) && chan_pad_supported(o, cin, cout, dt))
            return chan_pad_fwd_ws_bytes(o, cin, cout);
        return 0;
    }
    case SP_OP_WGRAD:
        if (conv_c1_supported(o, cin, cout, dt)) return wgrad_c1_ws_bytes(o, cout);
        if (wgrad_mfma_supported(o, cin, cout, dt)) return wgrad_mfma_ws_bytes(o, cin, cout);
        if (chan_pad_supported(o, cin, cout, dt)) return chan_pad_wgrad_ws_bytes(o, cin, cout);
        return wgrad_direct_ws_bytes(o, cin, cout);
    case SP_OP_UPCONV_WGRAD: {
        Geo c;
        if (make_coarse(o, &c) != SP_OK) return static_cast<size_t>(-1);
        return upconv2_wgrad_ws_bytes(o, c, cin, cout, dt);
    }
    case SP_OP_LOSS:
        return loss_supported(o, cin) ? loss_ws_bytes(o, cin) : static_cast<size_t>(-1);
    case SP_OP_POINTWISE_WGRAD:
        return pointwise_small_supported(o, cin, cout, dt) ? pointwise_small_wgrad_ws_bytes(o, cin, cout)
                                                           : wgrad_direct_ws_bytes(o, cin, cout, 1);
    default:
        return static_cast<size_t>(-1);
    }
}

const char *sp_strerror(int code) {
    switch (code) {
    case SP_OK: return "ok";
    case SP_EINVAL: return "invalid argument (null or misaligned pointer, non-positive size, overlap)";
    case SP_EGEOM: return "tile grid does not divide the volume, or a tile is thinner than the halo";
    case SP_EUNSUPPORTED: return "unsupported halo width, dtype or channel count";
    case SP_EWORKSPACE: return "workspace missing or too small";
    case SP_ELAUNCH: return "HIP error at launch (see sp_last_hip_error)";
    default: return "unknown error";
    }
}

int sp_last_hip_error(void) { return g_last_hip_error.load(); }

static int check_copy_args(const void *a, const void *b, const sp_geom_t *g, int c, sp_dtype_t dt,
                           Geo *o) {
    if (!a || !b) return SP_EINVAL;
    int rc = make_geo(g, o);
    if (rc != SP_OK) return rc;
    if (!chan_ok(c)) return SP_EINVAL;
    if (!dtype_ok(dt)) return SP_EUNSUPPORTED;
    if (!aligned16(a) || !aligned16(b)) return SP_EINVAL;
    return SP_OK;
}

int sp_partition(const void *vol, void *P, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream) {
    Geo o;
    int rc = check_copy_args(vol, P, g, c, dt, &o);
    if (rc != SP_OK) return rc;
    const size_t es = elem_size(dt);
    if (overlap(vol, static_cast<size_t>(o.ntiles) * o.int_vox * c * es, P,
                static_cast<size_t>(o.ntiles) * o.tile_vox * c * es))
        return SP_EINVAL;
    return launch_partition(vol, P, o, c, dt, false, static_cast<hipStream_t>(stream));
}

int sp_unpartition(const void *P, void *vol, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream) {
    Geo o;
    int rc = check_copy_args(P, vol, g, c, dt, &o);
    if (rc != SP_OK) return rc;
    const size_t es = elem_size(dt);
    if (overlap(vol, static_cast<size_t>(o.ntiles) * o.int_vox * c * es, P,
                static_cast<size_t>(o.ntiles) * o.tile_vox * c * es))
        return SP_EINVAL;
    return launch_partition(vol, const_cast<void *>(P), o, c, dt, true,
                            static_cast<hipStream_t>(stream));
}

int halo_pack(const void *P, void *msg, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream) {
    Geo o;
    int rc = check_copy_args(P, msg, g, c, dt, &o);
    if (rc != SP_OK) return rc;
    const size_t es = elem_size(dt);
    if (overlap(P, static_cast<size_t>(o.ntiles) * o.tile_vox * c * es, msg,
                static_cast<size_t>(o.ntiles) * o.msg_vox * c * es))
        return SP_EINVAL;
    return launch_halo_pack(P, msg, o, c, dt, g->opts, static_cast<hipStream_t>(stream));
}

int halo_unpack(void *P, const void *msg, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream) {
    Geo o;
    int rc = check_copy_args(P, msg, g, c, dt, &o);
    if (rc != SP_OK) return rc;
    const size_t es = elem_size(dt);
    if (overlap(P, static_cast<size_t>(o.ntiles) * o.tile_vox * c * es, msg,
                static_cast<size_t>(o.ntiles) * o.msg_vox * c * es))
        return SP_EINVAL;
    return launch_halo_unpack(P, msg, o, c, dt, g->opts, static_cast<hipStream_t>(stream));
}

int sp_halo_exchange(void *P, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream) {
    Geo o;
    int rc = check_copy_args(P, P, g, c, dt, &o);
    if (rc != SP_OK) return rc;
    return launch_halo_exchange(P, o, c, dt, g->opts, static_cast<hipStream_t>(stream));
}

static int check_conv_args(const void *a, const void *b, const void *c, const sp_geom_t *g, int cin,
                           int cout, sp_dtype_t dt, Geo *o) {
    if (!a || !b || !c) return SP_EINVAL;
    int rc = make_geo(g, o);
    if (rc != SP_OK) return rc;
    if (cin <= 0 || cout <= 0) return SP_EINVAL;
    if (!dtype_ok(dt) || !chan_ok(cin) || !chan_ok(cout)) return SP_EUNSUPPORTED;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c)) return SP_EINVAL;
    return SP_OK;
}

// forward kernels that can write the one-bit ReLU mask: the 3-D marching kernels and the one-input-channel layer
static bool fwd_bits_supported(const Geo &o, int cin, int cout, sp_dtype_t dt) {
    return conv_mfma_bits_supported(o, cin, cout, dt) ||
           (!conv_mfma_supported(o, cin, cout, dt) && o.grow == 0 && conv_c1_supported(o, cin, cout, dt));
}

static int fwd_impl(const void *Px, const void *w, const float *bias, void *Py, void *bits, const sp_geom_t *g,
                    int cin, int cout, sp_dtype_t dt, uint32_t flags, void *ws, size_t ws_bytes,
                    void *stream) {
    Geo o;
    int rc = check_conv_args(Px, w, Py, g, cin, cout, dt, &o);
    if (rc != SP_OK) return rc;
    if (flags & ~static_cast<uint32_t>(SP_FLAG_RELU)) return SP_EINVAL;
    const size_t es = elem_size(dt);
    const size_t pv = static_cast<size_t>(o.ntiles) * o.tile_vox;
    if (overlap(Px, pv * cin * es, Py, pv * cout * es)) return SP_EINVAL;
    const bool relu = flags & SP_FLAG_RELU;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool gather = g->opts & SP_HALO_GATHER;
    if (gather && !conv_mfma_gather_supported(o, cin, cout, dt)) return SP_EUNSUPPORTED;
    if (bits) {
        if (!relu) return SP_EINVAL;
        if (!fwd_bits_supported(o, cin, cout, dt)) return SP_EUNSUPPORTED;
        if ((reinterpret_cast<uintptr_t>(bits) & 3) || overlap(bits, pv * (cout / 32) * 4, Py, pv * cout * es) ||
            overlap(bits, pv * (cout / 32) * 4, Px, pv * cin * es))
            return SP_EINVAL;
    }
    if (conv_mfma_supported(o, cin, cout, dt)) {
        const size_t need = conv_mfma_ws_bytes(o, cin, cout);
        if (need && (!ws || ws_bytes < need || !aligned16(ws))) return SP_EWORKSPACE;
        return launch_conv_mfma(Px, w, bias, Py, o, cin, cout, relu, false, ws, s, nullptr, nullptr, gather, bits);
    }
    if (o.grow == 0 && conv_c1_supported(o, cin, cout, dt))
        return launch_conv_c1_fwd(shifted(Px, o, 1, dt), w, bias, shifted(Py, o, cout, dt), o, cout, relu, s,
                                  bits ? static_cast<char *>(bits) + interior_shift(o) * (cout / 32) * 4 : nullptr);
    // few input channels: zero-padded copies in the workspace, then the matrix-core kernel
    if (!conv_c1_supported(o, cin, cout, dt) && chan_pad_supported(o, cin, cout, dt)) {
        const size_t need = chan_pad_fwd_ws_bytes(o, cin, cout);
        if (!ws || ws_bytes < need || !aligned16(ws)) return SP_EWORKSPACE;
        return launch_conv_chan_pad_fwd(Px, w, bias, Py, o, cin, cout, relu, ws, s);
    }
    return launch_conv_direct(Px, w, bias, Py, o, cin, cout, dt, relu, false, s);
}

int conv3d_fwd(const void *Px, const void *w, const float *bias, void *Py, const sp_geom_t *g,
               int cin, int cout, sp_dtype_t dt, uint32_t flags, void *ws, size_t ws_bytes,
               void *stream) {
    return fwd_impl(Px, w, bias, Py, nullptr, g, cin, cout, dt, flags, ws, ws_bytes, stream);
}

int conv3d_fwd_bits(const void *Px, const void *w, const float *bias, void *Py, void *bits, const sp_geom_t *g,
                    int cin, int cout, sp_dtype_t dt, uint32_t flags, void *ws, size_t ws_bytes, void *stream) {
    if (!bits) return SP_EINVAL;
    return fwd_impl(Px, w, bias, Py, bits, g, cin, cout, dt, flags, ws, ws_bytes, stream);
}

static int dgrad_impl(const void *Pdz, const void *w, const void *Pmask, void *Pdx, const sp_geom_t *g, int cin,
                      int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream,
                      const void *bits = nullptr) {
    Geo o;
    int rc = check_conv_args(Pdz, w, Pdx, g, cin, cout, dt, &o);
    if (rc != SP_OK) return rc;
    const size_t es = elem_size(dt);
    const size_t pv = static_cast<size_t>(o.ntiles) * o.tile_vox;
    if (overlap(Pdz, pv * cout * es, Pdx, pv * cin * es)) return SP_EINVAL;
    if (Pmask && (!aligned16(Pmask) || overlap(Pmask, pv * cin * es, Pdx, pv * cin * es))) return SP_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the kernel's "input channels" are cout and its "output channels" are cin
    const bool gather = g->opts & SP_HALO_GATHER;
    if (gather && !conv_mfma_gather_supported(o, cout, cin, dt)) return SP_EUNSUPPORTED;
    if (bits) {
        if (!conv_mfma_bits_supported(o, cout, cin, dt)) return SP_EUNSUPPORTED;
        if ((reinterpret_cast<uintptr_t>(bits) & 3) || overlap(bits, pv * (cin / 32) * 4, Pdx, pv * cin * es))
            return SP_EINVAL;
    }
    if (conv_mfma_supported(o, cout, cin, dt)) {
        const size_t need = conv_mfma_ws_bytes(o, cout, cin);
        if (need && (!ws || ws_bytes < need || !aligned16(ws))) return SP_EWORKSPACE;
        return launch_conv_mfma(Pdz, w, nullptr, Pdx, o, cout, cin, false, true, ws, s, Pmask, nullptr, gather,
                                const_cast<void *>(bits));
    }
    return launch_conv_direct(Pdz, w, nullptr, Pdx, o, cout, cin, dt, false, true, s, 3, Pmask);
}

int conv3d_dgrad(const void *Pdz, const void *w, void *Pdx, const sp_geom_t *g, int cin, int cout,
                 sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream) {
    return dgrad_impl(Pdz, w, nullptr, Pdx, g, cin, cout, dt, ws, ws_bytes, stream);
}

int conv3d_dgrad_relu(const void *Pdz, const void *w, const void *Px, void *Pdx, const sp_geom_t *g, int cin,
                      int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream) {
    if (!Px) return SP_EINVAL;
    return dgrad_impl(Pdz, w, Px, Pdx, g, cin, cout, dt, ws, ws_bytes, stream);
}

int conv3d_dgrad_bits(const void *Pdz, const void *w, const void *bits, void *Pdx, const sp_geom_t *g, int cin,
                      int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream) {
    if (!bits) return SP_EINVAL;
    return dgrad_impl(Pdz, w, nullptr, Pdx, g, cin, cout, dt, ws, ws_bytes, stream, bits);
}

size_t sp_relu_bits_bytes(const sp_geom_t *g, int c) {
    Geo o;
    if (make_geo(g, &o) != SP_OK || c <= 0 || c % 32) return 0;
    return static_cast<size_t>(o.ntiles) * o.tile_vox * (c / 32) * 4;
}

int sp_relu_bits_supported(int op, const sp_geom_t *g, int cin, int cout, sp_dtype_t dt) {
    Geo o;
    if (make_geo(g, &o) != SP_OK || !chan_ok(cin) || !chan_ok(cout) || !dtype_ok(dt)) return 0;
    switch (op) {
    case SP_OP_FWD: return fwd_bits_supported(o, cin, cout, dt) ? 1 : 0;
    case SP_OP_DGRAD: return conv_mfma_bits_supported(o, cout, cin, dt) ? 1 : 0;     // channel roles swapped
    default: return 0;
    }
}

int sp_relu_bits(const void *Py, void *bits, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream) {
    if (!Py || !bits) return SP_EINVAL;
    Geo o;
    int rc = make_geo(g, &o);
    if (rc != SP_OK) return rc;
    if (c <= 0) return SP_EINVAL;
    if (dt != SP_BF16 || c % 32) return SP_EUNSUPPORTED;
    const size_t pv = static_cast<size_t>(o.ntiles) * o.tile_vox;
    if (!aligned16(Py) || (reinterpret_cast<uintptr_t>(bits) & 3) || overlap(Py, pv * c * 2, bits, pv * (c / 32) * 4))
        return SP_EINVAL;
    return launch_relu_bits(Py, bits, pv * (c / 32), static_cast<hipStream_t>(stream));
}

int conv3d_wgrad(const void *Px, const void *Pdz, float *dw, float *db, const sp_geom_t *g, int cin,
                 int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream) {
    Geo o;
    int rc = check_conv_args(Px, Pdz, dw, g, cin, cout, dt, &o);
    if (rc != SP_OK) return rc;
    if (db && (reinterpret_cast<uintptr_t>(db) & 3u)) return SP_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool gather = g->opts & SP_HALO_GATHER;
    if (gather && !wgrad_mfma_gather_supported(o, cin, cout, dt)) return SP_EUNSUPPORTED;
    const bool c1 = conv_c1_supported(o, cin, cout, dt);
    const bool mfma = !c1 && wgrad_mfma_supported(o, cin, cout, dt);
    const bool pad = !c1 && !mfma && chan_pad_supported(o, cin, cout, dt);
    const size_t need = c1 ? wgrad_c1_ws_bytes(o, cout)
                           : (mfma ? wgrad_mfma_ws_bytes(o, cin, cout)
                                   : (pad ? chan_pad_wgrad_ws_bytes(o, cin, cout) : wgrad_direct_ws_bytes(o, cin, cout)));
    if (need && (!ws || ws_bytes < need || !aligned16(ws))) return SP_EWORKSPACE;
    if (pad) return launch_wgrad_chan_pad(Px, Pdz, dw, db, o, cin, cout, dt, ws, s);
    if (c1) return launch_wgrad_c1(shifted(Px, o, 1, dt), shifted(Pdz, o, cout, dt), dw, db, o, cout, ws, s);
    if (mfma)
        return launch_wgrad_mfma(shifted(Px, o, cin, dt), shifted(Pdz, o, cout, dt), dw, db, o, cin, cout, ws, s, nullptr, 0,
                                 gather);
    return launch_wgrad_direct(Px, Pdz, dw, db, o, cin, cout, dt, ws, s);
}

int conv3d_wgrad_static(const void *Px, const void *Pdz, float *dw, float *db, const sp_geom_t *g, int cin,
                        int cout, sp_dtype_t dt, void *stream) {
    // every argument check of conv3d_wgrad that can fail does so before the scratch address is looked up
    Geo o;
    int rc = check_conv_args(Px, Pdz, dw, g, cin, cout, dt, &o);
    if (rc != SP_OK) return rc;
    const size_t need = sp_workspace_bytes(SP_OP_WGRAD, g, cin, cout, dt);
    if (need == static_cast<size_t>(-1)) return SP_EUNSUPPORTED;
    if (need > static_cast<size_t>(SP_STATIC_SCRATCH_BYTES)) return SP_EWORKSPACE;
    void *ws = nullptr;
    if ((rc = static_scratch(&ws)) != SP_OK) return rc;
    return conv3d_wgrad(Px, Pdz, dw, db, g, cin, cout, dt, ws, SP_STATIC_SCRATCH_BYTES, stream);
}

// ---- the same three passes on a channel-wise concatenation that is never materialised ----------------

static int check_pair(const void *a, int ca, const void *b, int cb, sp_dtype_t dt) {
    if (!a || !b) return SP_EINVAL;
    if (ca <= 0 || cb <= 0) return SP_EINVAL;
    if (dt != SP_BF16 || ca % 32 != 0 || cb % 32 != 0) return SP_EUNSUPPORTED;
    if (!aligned16(a) || !aligned16(b)) return SP_EINVAL;
    return SP_OK;
}

static int fwd2_impl(const void *Pxa, int ca, const void *Pxb, int cb, const void *w, const float *bias, void *Py,
                     void *bits, const sp_geom_t *g, int cout, sp_dtype_t dt, uint32_t flags, void *ws,
                     size_t ws_bytes, void *stream) {
    Geo o;
    int rc = check_conv_args(Pxa, w, Py, g, ca + cb, cout, dt, &o);
    if (rc != SP_OK) return rc;
    if ((rc = check_pair(Pxa, ca, Pxb, cb, dt)) != SP_OK) return rc;
    if (flags & ~static_cast<uint32_t>(SP_FLAG_RELU)) return SP_EINVAL;
    if (!conv_mfma_supported(o, ca + cb, cout, dt)) return SP_EUNSUPPORTED;
    const bool gather = g->opts & SP_HALO_GATHER;
    if (gather && !conv_mfma_gather_supported(o, ca + cb, cout, dt)) return SP_EUNSUPPORTED;
    const size_t pv = static_cast<size_t>(o.ntiles) * o.tile_vox;
    if (overlap(Pxa, pv * ca * 2, Py, pv * cout * 2) || overlap(Pxb, pv * cb * 2, Py, pv * cout * 2)) return SP_EINVAL;
    const size_t need = conv_mfma_ws_bytes(o, ca + cb, cout);
    if (need && (!ws || ws_bytes < need || !aligned16(ws))) return SP_EWORKSPACE;
    if (bits) {
        if (!(flags & SP_FLAG_RELU)) return SP_EINVAL;
        if (!conv_mfma_bits_supported(o, ca + cb, cout, dt)) return SP_EUNSUPPORTED;
        const size_t nb = pv * (cout / 32) * 4;
        if ((reinterpret_cast<uintptr_t>(bits) & 3) || overlap(bits, nb, Py, pv * cout * 2) ||
            overlap(bits, nb, Pxa, pv * ca * 2) || overlap(bits, nb, Pxb, pv * cb * 2))
            return SP_EINVAL;
    }
    const ConvSplit sp{Pxb, ca, nullptr, 0};
    return launch_conv_mfma(Pxa, w, bias, Py, o, ca + cb, cout, flags & SP_FLAG_RELU, false, ws,
                            static_cast<hipStream_t>(stream), nullptr, &sp, gather, bits);
}

int conv3d_fwd2(const void *Pxa, int ca, const void *Pxb, int cb, const void *w, const float *bias, void *Py,
                const sp_geom_t *g, int cout, sp_dtype_t dt, uint32_t flags, void *ws, size_t ws_bytes,
                void *stream) {
    return fwd2_impl(Pxa, ca, Pxb, cb, w, bias, Py, nullptr, g, cout, dt, flags, ws, ws_bytes, stream);
}

int conv3d_fwd2_bits(const void *Pxa, int ca, const void *Pxb, int cb, const void *w, const float *bias, void *Py,
                     void *bits, const sp_geom_t *g, int cout, sp_dtype_t dt, uint32_t flags, void *ws,
                     size_t ws_bytes, void *stream) {
    if (!bits) return SP_EINVAL;
    return fwd2_impl(Pxa, ca, Pxb, cb, w, bias, Py, bits, g, cout, dt, flags, ws, ws_bytes, stream);
}

int conv3d_dgrad2(const void *Pdz, const void *w, void *Pdxa, int ca, void *Pdxb, int cb, const sp_geom_t *g,
                  int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream) {
    Geo o;
    int rc = check_conv_args(Pdz, w, Pdxa, g, ca + cb, cout, dt, &o);
    if (rc != SP_OK) return rc;
    if ((rc = check_pair(Pdxa, ca, Pdxb, cb, dt)) != SP_OK) return rc;
    if (!conv_mfma_supported(o, cout, ca + cb, dt)) return SP_EUNSUPPORTED;
    const bool gather = g->opts & SP_HALO_GATHER;
    if (gather && !conv_mfma_gather_supported(o, cout, ca + cb, dt)) return SP_EUNSUPPORTED;
    const size_t pv = static_cast<size_t>(o.ntiles) * o.tile_vox;
    if (overlap(Pdz, pv * cout * 2, Pdxa, pv * ca * 2) || overlap(Pdz, pv * cout * 2, Pdxb, pv * cb * 2) ||
        overlap(Pdxa, pv * ca * 2, Pdxb, pv * cb * 2))
        return SP_EINVAL;
    const size_t need = conv_mfma_ws_bytes(o, cout, ca + cb);
    if (need && (!ws || ws_bytes < need || !aligned16(ws))) return SP_EWORKSPACE;
    const ConvSplit sp{nullptr, 0, Pdxb, ca};
    return launch_conv_mfma(Pdz, w, nullptr, Pdxa, o, cout, ca + cb, false, true, ws,
                            static_cast<hipStream_t>(stream), nullptr, &sp, gather);
}

int conv3d_wgrad2(const void *Pxa, int ca, const void *Pxb, int cb, const void *Pdz, float *dw, float *db,
                  const sp_geom_t *g, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream) {
    Geo o;
    int rc = check_conv_args(Pxa, Pdz, dw, g, ca + cb, cout, dt, &o);
    if (rc != SP_OK) return rc;
    if ((rc = check_pair(Pxa, ca, Pxb, cb, dt)) != SP_OK) return rc;
    if (db && (reinterpret_cast<uintptr_t>(db) & 3u)) return SP_EINVAL;
    if (!wgrad_mfma_supported(o, ca + cb, cout, dt)) return SP_EUNSUPPORTED;
    const bool gather = g->opts & SP_HALO_GATHER;
    if (gather && !wgrad_mfma_gather_supported(o, ca + cb, cout, dt)) return SP_EUNSUPPORTED;
    const size_t need = wgrad_mfma_ws_bytes(o, ca + cb, cout);
    if (!ws || ws_bytes < need || !aligned16(ws)) return SP_EWORKSPACE;
    return launch_wgrad_mfma(shifted(Pxa, o, ca, dt), shifted(Pdz, o, cout, dt), dw, db, o, ca + cb, cout, ws,
                             static_cast<hipStream_t>(stream), shifted(Pxb, o, cb, dt), ca, gather);
}

int sp_relu_bwd(const void *Pdy, const void *Py, void *Pdz, const sp_geom_t *g, int c, sp_dtype_t dt,
                void *stream) {
    Geo o;
    if (!Pdy || !Py || !Pdz) return SP_EINVAL;
    int rc = make_geo(g, &o);
    if (rc != SP_OK) return rc;
    if (!chan_ok(c)) return SP_EINVAL;
    if (!dtype_ok(dt)) return SP_EUNSUPPORTED;
    if (!aligned16(Pdy) || !aligned16(Py) || !aligned16(Pdz)) return SP_EINVAL;
    return launch_relu_bwd(Pdy, Py, Pdz, static_cast<size_t>(o.ntiles) * o.tile_vox * c, dt,
                           static_cast<hipStream_t>(stream));
}

// ---- U-Net glue ---------------------------------------------------------------------------------

static int check_glue(const void *a, const void *b, const void *c, const sp_geom_t *g, int c1, int c2,
                      sp_dtype_t dt, Geo *fine, Geo *coarse) {
    if (!a || !b || !c) return SP_EINVAL;
    int rc = make_geo(g, fine);
    if (rc != SP_OK) return rc;
    if (c1 <= 0 || c2 <= 0) return SP_EINVAL;
    if (!dtype_ok(dt) || !chan_ok(c1) || !chan_ok(c2)) return SP_EUNSUPPORTED;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c)) return SP_EINVAL;
    fine->grow = 0;            // these operations work on interiors only
    if (coarse) return make_coarse(*fine, coarse);
    return SP_OK;
}

int sp_maxpool2_fwd(const void *Px, void *Py, const sp_geom_t *gf, int c, sp_dtype_t dt, void *stream) {
    Geo f, k;
    int rc = check_glue(Px, Py, Py, gf, c, c, dt, &f, &k);
    if (rc != SP_OK) return rc;
    return launch_maxpool2(shifted(Px, f, c, dt), nullptr, shifted(Py, k, c, dt), f, k, c, dt, false,
                           static_cast<hipStream_t>(stream));
}

int sp_maxpool2_bwd(const void *Px, const void *Pdy, void *Pdx, const sp_geom_t *gf, int c, sp_dtype_t dt,
                    void *stream) {
    Geo f, k;
    int rc = check_glue(Px, Pdy, Pdx, gf, c, c, dt, &f, &k);
    if (rc != SP_OK) return rc;
    return launch_maxpool2(shifted(Px, f, c, dt), shifted(Pdy, k, c, dt), shifted(Pdx, f, c, dt), f, k, c, dt, true,
                           static_cast<hipStream_t>(stream));
}

int sp_maxpool2_bwd_join(const void *Px, const void *Pdy, const void *Pskip, void *Pdz, const sp_geom_t *gf, int c,
                         sp_dtype_t dt, void *stream) {
    Geo f, k;
    int rc = check_glue(Px, Pdy, Pdz, gf, c, c, dt, &f, &k);
    if (rc != SP_OK) return rc;
    if (!Pskip || !aligned16(Pskip)) return SP_EINVAL;
    const size_t bytes = static_cast<size_t>(f.ntiles) * f.tile_vox * c * elem_size(dt);
    if (overlap(Px, bytes, Pdz, bytes)) return SP_EINVAL;
    if (Pskip != Pdz && overlap(Pskip, bytes, Pdz, bytes)) return SP_EINVAL;
    return launch_maxpool2(shifted(Px, f, c, dt), shifted(Pdy, k, c, dt), shifted(Pdz, f, c, dt), f, k, c, dt, true,
                           static_cast<hipStream_t>(stream), shifted(Pskip, f, c, dt));
}

int sp_upconv2_fwd(const void *Px, const void *u, const float *bias, void *Py, const sp_geom_t *gf, int cin,
                   int cout, sp_dtype_t dt, void *stream) {
    Geo f, k;
    int rc = check_glue(Px, u, Py, gf, cin, cout, dt, &f, &k);
    if (rc != SP_OK) return rc;
    return launch_upconv2_fwd(shifted(Px, k, cin, dt), u, bias, shifted(Py, f, cout, dt), f, k, cin, cout, dt,
                              static_cast<hipStream_t>(stream));
}

int sp_upconv2_dgrad(const void *Pdy, const void *u, void *Pdx, const sp_geom_t *gf, int cin, int cout,
                     sp_dtype_t dt, void *stream) {
    Geo f, k;
    int rc = check_glue(Pdy, u, Pdx, gf, cin, cout, dt, &f, &k);
    if (rc != SP_OK) return rc;
    return launch_upconv2_dgrad(shifted(Pdy, f, cout, dt), u, shifted(Pdx, k, cin, dt), f, k, cin, cout, dt,
                                static_cast<hipStream_t>(stream));
}

int sp_upconv2_wgrad(const void *Px, const void *Pdy, float *du, float *db, const sp_geom_t *gf, int cin,
                     int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream) {
    Geo f, k;
    int rc = check_glue(Px, Pdy, du, gf, cin, cout, dt, &f, &k);
    if (rc != SP_OK) return rc;
    const size_t need = upconv2_wgrad_ws_bytes(f, k, cin, cout, dt);
    if (!ws || ws_bytes < need || !aligned16(ws)) return SP_EWORKSPACE;
    return launch_upconv2_wgrad(shifted(Px, k, cin, dt), shifted(Pdy, f, cout, dt), du, db, f, k, cin, cout, dt, ws,
                                static_cast<hipStream_t>(stream));
}

int sp_pointwise_fwd(const void *Px, const void *p, const float *bias, void *Py, const sp_geom_t *g, int cin,
                     int cout, sp_dtype_t dt, uint32_t flags, void *stream) {
    Geo o;
    int rc = check_glue(Px, p, Py, g, cin, cout, dt, &o, nullptr);
    if (rc != SP_OK) return rc;
    if (flags & ~static_cast<uint32_t>(SP_FLAG_RELU)) return SP_EINVAL;
    if (pointwise_small_supported(o, cin, cout, dt))
        return launch_pointwise_small_fwd(shifted(Px, o, cin, dt), p, bias, shifted(Py, o, cout, dt), o, cin, cout,
                                          flags & SP_FLAG_RELU, static_cast<hipStream_t>(stream));
    return launch_conv_direct(Px, p, bias, Py, o, cin, cout, dt, flags & SP_FLAG_RELU, false,
                              static_cast<hipStream_t>(stream), 1);
}

static int pointwise_dgrad_impl(const void *Pdy, const void *p, const void *Pmask, void *Pdx, const sp_geom_t *g,
                                int cin, int cout, sp_dtype_t dt, void *stream) {
    Geo o;
    int rc = check_glue(Pdy, p, Pdx, g, cin, cout, dt, &o, nullptr);
    if (rc != SP_OK) return rc;
    if (Pmask) {
        const size_t bytes = static_cast<size_t>(o.ntiles) * o.tile_vox * cin * elem_size(dt);
        if (!aligned16(Pmask) || overlap(Pmask, bytes, Pdx, bytes)) return SP_EINVAL;
    }
    if (pointwise_small_supported(o, cin, cout, dt))
        return launch_pointwise_small_dgrad(shifted(Pdy, o, cout, dt), p, shifted(Pdx, o, cin, dt), o, cin, cout,
                                            static_cast<hipStream_t>(stream), shifted(Pmask, o, cin, dt));
    return launch_conv_direct(Pdy, p, nullptr, Pdx, o, cout, cin, dt, false, true,
                              static_cast<hipStream_t>(stream), 1, Pmask);
}

int sp_pointwise_dgrad(const void *Pdy, const void *p, void *Pdx, const sp_geom_t *g, int cin, int cout,
                       sp_dtype_t dt, void *stream) {
    return pointwise_dgrad_impl(Pdy, p, nullptr, Pdx, g, cin, cout, dt, stream);
}

int sp_pointwise_dgrad_relu(const void *Pdy, const void *p, const void *Px, void *Pdx, const sp_geom_t *g, int cin,
                            int cout, sp_dtype_t dt, void *stream) {
    if (!Px) return SP_EINVAL;
    return pointwise_dgrad_impl(Pdy, p, Px, Pdx, g, cin, cout, dt, stream);
}

int sp_pointwise_wgrad(const void *Px, const void *Pdy, float *dp, float *db, const sp_geom_t *g, int cin,
                       int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream) {
    Geo o;
    int rc = check_glue(Px, Pdy, dp, g, cin, cout, dt, &o, nullptr);
    if (rc != SP_OK) return rc;
    const bool small = pointwise_small_supported(o, cin, cout, dt);
    const size_t need = small ? pointwise_small_wgrad_ws_bytes(o, cin, cout) : wgrad_direct_ws_bytes(o, cin, cout, 1);
    if (!ws || ws_bytes < need || !aligned16(ws)) return SP_EWORKSPACE;
    if (small)
        return launch_pointwise_small_wgrad(shifted(Px, o, cin, dt), shifted(Pdy, o, cout, dt), dp, db, o, cin, cout, ws,
                                            static_cast<hipStream_t>(stream));
    return launch_wgrad_direct(Px, Pdy, dp, db, o, cin, cout, dt, ws, static_cast<hipStream_t>(stream), 1);
}

int sp_pointwise_bwd_relu(const void *Px, const void *Pdy, const void *p, void *Pdx, float *dp, float *db,
                          const sp_geom_t *g, int cin, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes,
                          void *stream) {
    if (!p || !Pdx) return SP_EINVAL;
    Geo o;
    int rc = check_glue(Px, Pdy, dp, g, cin, cout, dt, &o, nullptr);
    if (rc != SP_OK) return rc;
    const size_t bytes = static_cast<size_t>(o.ntiles) * o.tile_vox * cin * elem_size(dt);
    if (!aligned16(Pdx) || overlap(Px, bytes, Pdx, bytes)) return SP_EINVAL;
    if (!pointwise_small_supported(o, cin, cout, dt)) {      // the two passes one after the other
        rc = sp_pointwise_dgrad_relu(Pdy, p, Px, Pdx, g, cin, cout, dt, stream);
        if (rc != SP_OK) return rc;
        return sp_pointwise_wgrad(Px, Pdy, dp, db, g, cin, cout, dt, ws, ws_bytes, stream);
    }
    if (!ws || ws_bytes < pointwise_small_wgrad_ws_bytes(o, cin, cout) || !aligned16(ws)) return SP_EWORKSPACE;
    return launch_pointwise_small_wgrad(shifted(Px, o, cin, dt), shifted(Pdy, o, cout, dt), dp, db, o, cin, cout, ws,
                                        static_cast<hipStream_t>(stream), p, shifted(Pdx, o, cin, dt));
}

int sp_dice_ce_loss(const void *Plogits, const void *Plabels, void *Pdlogits, float *loss, float *stats,
                    const sp_geom_t *g, int classes, sp_dtype_t dt, float w_dice, float w_ce, float eps, void *ws,
                    size_t ws_bytes, void *stream) {
    if (!Plogits || !Plabels || (!Pdlogits && !loss && !stats)) return SP_EINVAL;
    Geo o;
    int rc = make_geo(g, &o);
    if (rc != SP_OK) return rc;
    if (!dtype_ok(dt)) return SP_EUNSUPPORTED;
    if (classes < 2) return SP_EINVAL;
    if (!loss_supported(o, classes)) return SP_EUNSUPPORTED;
    if (!aligned16(Plogits) || !aligned16(Plabels) || (Pdlogits && !aligned16(Pdlogits))) return SP_EINVAL;
    if ((loss && (reinterpret_cast<uintptr_t>(loss) & 3u)) || (stats && (reinterpret_cast<uintptr_t>(stats) & 3u)))
        return SP_EINVAL;
    if (!(eps >= 0.f) || !(w_dice >= 0.f) || !(w_ce >= 0.f)) return SP_EINVAL;
    const size_t need = loss_ws_bytes(o, classes);
    if (!ws || ws_bytes < need || !aligned16(ws)) return SP_EWORKSPACE;
    return launch_loss(shifted(Plogits, o, classes, dt), shifted(Plabels, o, 1, dt), shifted(Pdlogits, o, classes, dt),
                       loss, stats, o, classes, dt, w_dice, w_ce, eps, ws, static_cast<hipStream_t>(stream));
}

int sp_concat(const void *Pa, int ca, const void *Pb, int cb, void *Pout, const sp_geom_t *g, sp_dtype_t dt,
              void *stream) {
    Geo o;
    int rc = check_glue(Pa, Pb, Pout, g, ca, cb, dt, &o, nullptr);
    if (rc != SP_OK) return rc;
    return launch_concat(Pa, ca, Pb, cb, Pout, static_cast<size_t>(o.ntiles) * o.tile_vox, dt, false,
                         static_cast<hipStream_t>(stream));
}

int sp_split(const void *Pin, void *Pa, int ca, void *Pb, int cb, const sp_geom_t *g, sp_dtype_t dt,
             void *stream) {
    Geo o;
    int rc = check_glue(Pin, Pa, Pb, g, ca, cb, dt, &o, nullptr);
    if (rc != SP_OK) return rc;
    return launch_concat(Pa, ca, Pb, cb, const_cast<void *>(Pin), static_cast<size_t>(o.ntiles) * o.tile_vox,
                         dt, true, static_cast<hipStream_t>(stream));
}

int sp_add(const void *Pa, const void *Pb, void *Pout, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream) {
    Geo o;
    int rc = check_glue(Pa, Pb, Pout, g, c, c, dt, &o, nullptr);
    if (rc != SP_OK) return rc;
    return launch_add(Pa, Pb, Pout, static_cast<size_t>(o.ntiles) * o.tile_vox * c, dt,
                      static_cast<hipStream_t>(stream));
}

}  // extern "C"
