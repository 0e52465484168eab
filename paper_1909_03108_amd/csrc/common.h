// Internal declarations shared by the HIP sources of libsp3d (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <type_traits>
#include "sp3d.h"

namespace sp3d {

// Stores of results that nothing reads again before they have left every cache (whole activations and gradients
// of a layer, gigabytes against 4 MB of L2 per XCD), written non-temporally.  Only where a wave's store covers whole
// runs of memory, 16 bytes per lane and neighbouring lanes side by side: first layer forward at 512^3 2.39 -> 1.91
// ms, transposed convolution forward 2.61 -> 2.34, max-pool forward 1.75 -> 1.63, the 1x1x1 head's data gradient
// 3.70 -> 3.60.  8-byte pieces that lie a record or more apart need the cache to be put together: the same kind of
// store made the transposed convolution's data gradient 2.5 times slower.
#if defined(__HIPCC__)
typedef uint32_t st_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void st_stream16(void *p, uint4 v) {
    __builtin_nontemporal_store(st_u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<st_u32x4 *>(p));
}
#endif

// Geometry in the form the kernels use: tile extents, padded extents and strides in voxels.
struct Geo {
    int n, gd, gh, gw;       // batch and tile grid
    int td, th, tw;          // tile extents
    int pd, ph, pw;          // padded tile extents (t + 2*halo)
    int halo;
    int grow;                // conv3d_fwd / conv3d_dgrad: output box = interior grown by this many voxels
                             // towards every neighbouring tile (0 <= grow < halo); other operations ignore it
    int flat;                // 1: 2-D variant, D is a stack of independent slices (kernel / window extent 1 along D)
    int ntiles;              // n * gd * gh * gw
    long long tile_vox;      // pd * ph * pw   (voxels per padded tile)
    long long int_vox;       // td * th * tw   (interior voxels per tile)
    long long msg_vox;       // tile_vox - int_vox (margin voxels per tile)
};

int make_geo(const sp_geom_t *g, Geo *out);       // SP_OK or error code
// Kernels that touch tile interiors only are written for a one-voxel margin: interior voxel (i, j, k) at
// padded coordinates (i + 1, j + 1, k + 1), strides ph * pw and pw.  A tensor with a wider margin is handed
// to them through this offset (in voxels) on its base pointer: the strides stay those of the real layout.
inline long long interior_shift(const Geo &g) { return (g.halo - 1) * (1LL * g.ph * g.pw + g.pw + 1); }
template <typename T> inline T *shifted(T *p, const Geo &g, int c, sp_dtype_t dt) {
    typedef typename std::conditional<std::is_const<T>::value, const char, char>::type B;
    return p ? reinterpret_cast<T *>(reinterpret_cast<B *>(p) + interior_shift(g) * c * (dt == SP_BF16 ? 2 : 4)) : p;
}
int record_hip(hipError_t e);                      // stores e, returns SP_ELAUNCH if e != success
__host__ __device__ inline int grow_d(const Geo &g) { return g.flat ? 0 : g.grow; }      // growth of a convolution's output box along D
__host__ __device__ inline int taps_of(const Geo &g) { return g.flat ? 9 : 27; }          // taps of the 3x3(x3) kernel
inline size_t elem_size(sp_dtype_t dt) { return dt == SP_BF16 ? 2 : 4; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// One of the 26 halo regions, in message order.
struct Region {
    int ext[3];      // extents (d,h,w) of the region
    int send[3];     // origin of the sent box in padded coordinates of the sending tile
    int recv[3];     // origin of the margin box in padded coordinates of the receiving tile
    int delta[3];    // direction
    int opposite;    // index of the region with direction -delta
    long long off;   // voxel offset of the region inside a tile's message
};
struct RegionTable {
    Region r[26];
};
void make_regions(const Geo &g, RegionTable *t);

// launchers implemented in the kernel sources -------------------------------------------------
int launch_partition(const void *vol, void *P, const Geo &g, int c, sp_dtype_t dt, bool inverse,
                     hipStream_t s);
// border: the SP_HALO_* flags of the call's geometry
int launch_halo_pack(const void *P, void *msg, const Geo &g, int c, sp_dtype_t dt, int border, hipStream_t s);
int launch_halo_unpack(void *P, const void *msg, const Geo &g, int c, sp_dtype_t dt, int border, hipStream_t s);
int launch_halo_exchange(void *P, const Geo &g, int c, sp_dtype_t dt, int border, hipStream_t s);
int launch_relu_bwd(const void *dy, const void *y, void *dz, size_t elems, sp_dtype_t dt,
                    hipStream_t s);
// one-bit ReLU mask of a bf16 tensor: `blocks` records of 32 channels -> one 32-bit word each
int launch_relu_bits(const void *y, void *bits, size_t blocks, hipStream_t s);

// ks = kernel extent per axis (3, or 1 for the 1x1x1 convolution); mask (optional): tensor laid out like Pout,
// results are zeroed where it is not positive
int launch_conv_direct(const void *Pin, const void *w, const float *bias, void *Pout, const Geo &g,
                       int cin, int cout, sp_dtype_t dt, bool relu, bool dgrad, hipStream_t s, int ks = 3,
                       const void *mask = nullptr);
size_t wgrad_direct_ws_bytes(const Geo &g, int cin, int cout, int ks = 3);
int launch_wgrad_direct(const void *Px, const void *Pdz, float *dw, float *db, const Geo &g,
                        int cin, int cout, sp_dtype_t dt, void *ws, hipStream_t s, int ks = 3);

// U-Net glue (glue_kernels.hip).  gf = geometry of the fine (higher-resolution) volume.
int make_coarse(const Geo &gf, Geo *gc);     // SP_OK, or SP_EGEOM if a tile extent is odd
// backward with Pskip: Pout = [Px > 0] * (maxpool_bwd(Px, Pdy) + Pskip)   (Pskip may be Pout)
int launch_maxpool2(const void *Px, const void *Pdy, void *Pout, const Geo &gf, const Geo &gc, int c,
                    sp_dtype_t dt, bool backward, hipStream_t s, const void *Pskip = nullptr);
int launch_upconv2_fwd(const void *Px, const void *u, const float *bias, void *Py, const Geo &gf,
                       const Geo &gc, int cin, int cout, sp_dtype_t dt, hipStream_t s);
int launch_upconv2_dgrad(const void *Pdy, const void *u, void *Pdx, const Geo &gf, const Geo &gc, int cin,
                         int cout, sp_dtype_t dt, hipStream_t s);
size_t upconv2_wgrad_ws_bytes(const Geo &gf, const Geo &gc, int cin, int cout, sp_dtype_t dt);
int launch_upconv2_wgrad(const void *Px, const void *Pdy, float *du, float *db, const Geo &gf, const Geo &gc,
                         int cin, int cout, sp_dtype_t dt, void *ws, hipStream_t s);
// matrix-core variants of the transposed convolution (upconv_mfma.hip); bf16, channels in multiples of 32
bool upconv_mfma_supported(const Geo &gf, const Geo &gc, int cin, int cout, sp_dtype_t dt);
int launch_upconv_fwd_mfma(const void *Px, const void *u, const float *bias, void *Py, const Geo &gf,
                           const Geo &gc, int cin, int cout, hipStream_t s);
int launch_upconv_dgrad_mfma(const void *Pdy, const void *u, void *Pdx, const Geo &gf, const Geo &gc, int cin,
                             int cout, hipStream_t s);
size_t upconv_wgrad_mfma_ws_bytes(const Geo &gc, int cin, int cout);
int launch_upconv_wgrad_mfma(const void *Px, const void *Pdy, float *du, float *db, const Geo &gf, const Geo &gc,
                             int cin, int cout, void *ws, hipStream_t s);
// 1x1x1 convolution with at most 4 output channels (segmentation head), bf16 (glue_kernels.hip)
bool pointwise_small_supported(const Geo &g, int cin, int cout, sp_dtype_t dt);
int launch_pointwise_small_fwd(const void *Px, const void *p, const float *bias, void *Py, const Geo &g, int cin,
                               int cout, bool relu, hipStream_t s);
// Pmask (optional): laid out like Pdx; results are zeroed where it is not positive
int launch_pointwise_small_dgrad(const void *Pdy, const void *p, void *Pdx, const Geo &g, int cin, int cout,
                                 hipStream_t s, const void *Pmask = nullptr);
size_t pointwise_small_wgrad_ws_bytes(const Geo &g, int cin, int cout);
// (p, Pdx: null, or the weights and the output of the masked data gradient computed in the same pass)
int launch_pointwise_small_wgrad(const void *Px, const void *Pdy, float *dp, float *db, const Geo &g, int cin,
                                 int cout, void *ws, hipStream_t s, const void *p = nullptr, void *Pdx = nullptr);
// soft Dice + cross-entropy over the class logits and its gradient (loss_kernels.hip)
bool loss_supported(const Geo &g, int classes);
size_t loss_ws_bytes(const Geo &g, int classes);
int launch_loss(const void *Pz, const void *Plab, void *Pdz, float *loss, float *stats, const Geo &g, int classes,
                sp_dtype_t dt, float w_dice, float w_ce, float eps, void *ws, hipStream_t s);
int launch_add(const void *Pa, const void *Pb, void *Pout, size_t elems, sp_dtype_t dt, hipStream_t s);
int launch_concat(const void *Pa, int ca, const void *Pb, int cb, void *Pc, size_t voxels, sp_dtype_t dt,
                  bool split, hipStream_t s);

int launch_reduce_partials(const float *part, float *out, int nparts, long long n, hipStream_t s);

bool conv_mfma_supported(const Geo &g, int cin, int cout, sp_dtype_t dt);
size_t conv_mfma_ws_bytes(const Geo &g, int cin, int cout);
// Channel-wise concatenation without a copy: the kernel's input channels [in_ca, cin) may live in a second
// tensor in2 (cin - in_ca channels per voxel, Pin then has in_ca), and its output channels [out_ca, cout) may
// go to a second tensor out2 (cout - out_ca per voxel, Pout then has out_ca).  Null pointers = not split.
struct ConvSplit {
    const void *in2; int in_ca;
    void *out2; int out_ca;
};
// mask (optional, data gradient): tensor laid out like Pout; results are zeroed where it is not positive
// gather: margin voxels that have a neighbour tile are read from that tile's interior (SP_HALO_GATHER)
// bits (optional): the one-bit ReLU mask (layout: sp3d.h, sp_relu_bits) - read by a data gradient instead of a
// mask tensor (zero where the bit is clear), written by a forward pass with ReLU (bit = result positive)
bool conv_mfma_gather_supported(const Geo &g, int cin, int cout, sp_dtype_t dt);
bool conv_mfma_bits_supported(const Geo &g, int cin, int cout, sp_dtype_t dt);
int launch_conv_mfma(const void *Pin, const void *w, const float *bias, void *Pout, const Geo &g,
                     int cin, int cout, bool relu, bool dgrad, void *ws, hipStream_t s,
                     const void *mask = nullptr, const ConvSplit *split = nullptr, bool gather = false,
                     void *bits = nullptr);

// wide layers on few voxels: output-stationary implicit GEMM on the packed weights (conv_gemm.hip);
// launch_conv_mfma hands such layers over after packing
bool conv_gemm_preferred(const Geo &g, int ki, int ko);
int launch_conv_gemm(const void *Pin, const void *wpack, const float *bias, void *Pout, const Geo &g, int ki, int ko,
                     bool relu, hipStream_t s, const void *mask, const ConvSplit *split);

// single-input-channel first layer (conv_c1.hip)
bool conv_c1_supported(const Geo &g, int cin, int cout, sp_dtype_t dt);
// bits (optional, with relu): also writes the one-bit ReLU mask of the result (pointer shifted like Py)
int launch_conv_c1_fwd(const void *Px, const void *w, const float *bias, void *Py, const Geo &g, int cout,
                       bool relu, hipStream_t s, void *bits = nullptr);
size_t wgrad_c1_ws_bytes(const Geo &g, int cout);
int launch_wgrad_c1(const void *Px, const void *Pdz, float *dw, float *db, const Geo &g, int cout, void *ws,
                    hipStream_t s);

bool wgrad_mfma_supported(const Geo &g, int cin, int cout, sp_dtype_t dt);
size_t wgrad_mfma_ws_bytes(const Geo &g, int cin, int cout);
// Px2 (optional): the input channels [ca, cin) live in a second tensor of cin - ca channels per voxel
// gather: margin voxels of x that have a neighbour tile are read from that tile's interior (SP_HALO_GATHER)
bool wgrad_mfma_gather_supported(const Geo &g, int cin, int cout, sp_dtype_t dt);
int launch_wgrad_mfma(const void *Px, const void *Pdz, float *dw, float *db, const Geo &g,
                      int cin, int cout, void *ws, hipStream_t s, const void *Px2 = nullptr, int ca = 0,
                      bool gather = false);

// few input channels (not a multiple of 32) on the matrix cores through zero-padded copies (chan_pad.hip)
bool chan_pad_supported(const Geo &g, int cin, int cout, sp_dtype_t dt);
size_t chan_pad_fwd_ws_bytes(const Geo &g, int cin, int cout);
size_t chan_pad_wgrad_ws_bytes(const Geo &g, int cin, int cout);
int launch_conv_chan_pad_fwd(const void *Px, const void *w, const float *bias, void *Py, const Geo &g, int cin,
                             int cout, bool relu, void *ws, hipStream_t s);
int launch_wgrad_chan_pad(const void *Px, const void *Pdz, float *dw, float *db, const Geo &g, int cin, int cout,
                          sp_dtype_t dt, void *ws, hipStream_t s);

// Division of a 32-bit index by a launch-time constant without the ~25-instruction software divide:
// multiply-high by a precomputed reciprocal, with the one-bit-wider "add" form where the 32-bit
// reciprocal is not exact (Granlund & Montgomery, "Division by invariant integers using
// multiplication").  Exact for every 32-bit numerator.
struct FastDiv {
    uint32_t d, magic, shift, add;
};
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f{d, 0, 0, 0};
    if (d == 0) return f;                                      // (no divisor: callers never divide by it)
    uint32_t L = 31;
    while (!((d >> L) & 1)) --L;                               // floor(log2 d), d >= 1
    if ((d & (d - 1)) == 0) { f.shift = L; return f; }         // power of two: plain shift
    const uint64_t two = 1ull << (32 + L);
    uint64_t m = two / d;
    const uint64_t rem = two - m * d;
    if (d - rem < (1ull << L)) { f.magic = static_cast<uint32_t>(m + 1); f.shift = L; return f; }
    m = 2 * m + (2 * rem >= d ? 1 : 0);                        // one more quotient bit
    f.magic = static_cast<uint32_t>(m + 1); f.shift = L; f.add = 1;
    return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f) {
    if (!f.magic) return n >> f.shift;
    uint32_t q = __umulhi(n, f.magic);
    if (f.add) q = ((n - q) >> 1) + q;
    return q >> f.shift;
}
__device__ __forceinline__ uint32_t fmod_(uint32_t n, uint32_t q, const FastDiv &f) { return n - q * f.d; }

// device helpers ------------------------------------------------------------------------------
// Output box of a convolution on one tile: the interior, grown by g.grow voxels on every side where the tile
// has a neighbour in the grid (so the box never leaves the volume: beyond the volume border an activation is
// zero padding, not a convolution result).  org = voxel offset, inside the padded tile, of the corner one
// voxel before the box on every axis: a kernel written for a one-voxel margin sees the box as the interior
// of a padded tile that starts there.
struct TileBox {
    int bd, bh, bw;
    long long org;
};
__device__ __forceinline__ TileBox tile_box(const Geo &g, int tile) {
    TileBox b;
    int ld = g.halo, lh = g.halo, lw = g.halo;
    b.bd = g.td; b.bh = g.th; b.bw = g.tw;
    if (g.grow > 0) {
        const int tc = tile % g.gw, t1 = tile / g.gw;
        const int tb = t1 % g.gh, ta = (t1 / g.gh) % g.gd;
        if (!g.flat) {          // slices of the 2-D variant do not interact: nothing to grow along D
            if (ta > 0) { ld -= g.grow; b.bd += g.grow; }
            if (ta < g.gd - 1) b.bd += g.grow;
        }
        if (tb > 0) { lh -= g.grow; b.bh += g.grow; }
        if (tb < g.gh - 1) b.bh += g.grow;
        if (tc > 0) { lw -= g.grow; b.bw += g.grow; }
        if (tc < g.gw - 1) b.bw += g.grow;
    }
    b.org = (1LL * (ld - 1) * g.ph + lh - 1) * g.pw + lw - 1;
    return b;
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

}  // namespace sp3d
