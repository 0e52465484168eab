// bf16 2x2x2 stride-2 transposed convolution (the up-sampling step of the U-Net decoder) on the gfx950
// matrix cores: forward and data gradient.  Both are per-voxel channel mixes, i.e. plain GEMMs whose long
// dimension is the voxel index:
//
//   forward   y[2v + t][co] = bias[co] + sum_ci u[t][ci][co] * x[v][ci]          K = Cin,      8 taps t
//   dgrad     dx[v][ci]     = sum_t sum_co u[t][ci][co] * dy[2v + t][co]         K = 8 * Cout
//
// v_mfma_f32_32x32x16_bf16 with the weights as the A operand (rows = output channels of the product) and
// 32 consecutive coarse voxels of one W row as the B operand (columns): NDHWC keeps a voxel's channels
// contiguous, so a B fragment is one 16-byte global load per lane and needs no LDS.  The weight fragments
// of a workgroup's channel block are built once in LDS (forward: transposed on the way in, because the
// product reduces over ci while u is stored [ci][co]; dgrad: already in fragment order) and re-read for
// every 32-voxel segment.  The result lane layout - lane l holds voxel l % 32 and channels
// 8*(i/4) + 4*(l/32) + i%4 - gives 8-byte stores.  Both kernels are bound by HBM traffic, not by the
// matrix cores; a workgroup is persistent and its 8 waves walk over segments independently.
#include "common.h"

namespace sp3d {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kT = 512;          // 8 waves, 2 per SIMD
constexpr int C = 32;            // channel block = MFMA rows
constexpr int SEG = 32;          // voxels per segment = MFMA columns
constexpr int kMaxFragKB = 128;  // LDS spent on weight fragments (1 KB each)
constexpr int kGroups = 256;     // workgroups per launch: one per CU

struct UpArgs {
    const uint16_t *in;      // forward: x (coarse);  dgrad: dy (fine)
    const uint16_t *u;       // [8][cin][cout]
    const float *bias;       // forward only, may be null
    uint16_t *out;           // forward: y (fine);  dgrad: dx (coarse)
    Geo gf, gc;
    int cin, cout;
    int nblk;                // channel blocks of the output handled by different workgroups
    int wpb;                 // workgroups per channel block
    int nseg;                // segments per coarse W row
    int nitems;              // segments in total
};

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    union { bf16x2 v; uint32_t u; } r;
    r.v = __builtin_convertvector(f32x2{a, b}, bf16x2);
    return r.u;
}

struct Item { int tile, d, h, w0; };
__device__ __forceinline__ Item decode_item(int item, const UpArgs &a) {
    Item o;
    o.w0 = (item % a.nseg) * SEG;
    int t = item / a.nseg;
    o.h = t % a.gc.th; t /= a.gc.th;
    o.d = t % a.gc.td;
    o.tile = t / a.gc.td;
    return o;
}
// padded voxel index of interior voxel (d, h, w) of a tile
__device__ __forceinline__ size_t pvox(const Geo &g, int tile, int d, int h, int w) {
    return static_cast<size_t>(tile) * g.tile_vox + (static_cast<size_t>(d + 1) * g.ph + h + 1) * g.pw + w + 1;
}

// ---- forward -----------------------------------------------------------------------------------------
// NKS = Cin / 16 reduction steps.  LDS: fragment (tap, ks) at (tap * NKS + ks) KB; lane l of it holds
// u[tap][16 ks + 8 (l/32) + j][32 cb + l % 32], j = 0..7.
template <int NKS>
__global__ __launch_bounds__(kT) void upconv_fwd_mfma_kernel(UpArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int cb = blockIdx.x % a.nblk, sub = blockIdx.x / a.nblk;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int CIN = 16 * NKS;
    // weights: 16-byte pieces (8 output channels of one (tap, ci)) scattered to the 8 lanes that own them
    for (int e = tid; e < 8 * CIN * 4; e += kT) {
        const int c8 = e & 3, ci = (e >> 2) % CIN, tap = (e >> 2) / CIN;
        const uint4 v = *reinterpret_cast<const uint4 *>(a.u + (static_cast<size_t>(tap) * CIN + ci) * a.cout +
                                                         C * cb + 8 * c8);
        char *dst = lds + (tap * NKS + (ci >> 4)) * 1024 + ((ci >> 3) & 1) * 512 + (ci & 7) * 2 + 8 * c8 * 16;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 8; ++j)
            *reinterpret_cast<uint16_t *>(dst + j * 16) = static_cast<uint16_t>(w[j >> 1] >> (16 * (j & 1)));
    }
    __syncthreads();

    const int m = lane & 31, kh = lane >> 5;
    float bv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) bv[i] = a.bias ? a.bias[C * cb + 8 * (i >> 2) + 4 * kh + (i & 3)] : 0.f;

    // Items are taken two at a time so that the x fragments of the next one are in flight while the current
    // one is multiplied (the named buffers b0 / b1 swap roles without register copies).
    const int stride = a.wpb * (kT / 64);
    bf16x8 b0[NKS], b1[NKS];
    auto fetch = [&](int item, bf16x8 (&b)[NKS]) {
        if (item >= a.nitems) return;
        const Item o = decode_item(item, a);
        const int w = min(o.w0 + m, a.gc.tw - 1);
        const uint16_t *px = a.in + pvox(a.gc, o.tile, o.d, o.h, w) * CIN + 8 * kh;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) b[ks] = *reinterpret_cast<const bf16x8 *>(px + 16 * ks);
    };
    auto compute = [&](int item, const bf16x8 (&b)[NKS]) {
        const Item o = decode_item(item, a);
        const int w = o.w0 + m;
        const bool ok = w < a.gc.tw;
#pragma unroll 1
        for (int tap = 0; tap < 8; ++tap) {
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = bv[i];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const bf16x8 af = *reinterpret_cast<const bf16x8 *>(lds + (tap * NKS + ks) * 1024 + lane * 16);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b[ks], acc, 0, 0, 0);
            }
            if (ok) {
                uint16_t *py = a.out + pvox(a.gf, o.tile, 2 * o.d + (tap >> 2), 2 * o.h + ((tap >> 1) & 1),
                                            2 * w + (tap & 1)) * a.cout + C * cb + 4 * kh;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2 *>(py + 8 * q) = make_uint2(pack2(acc[4 * q], acc[4 * q + 1]),
                                                                       pack2(acc[4 * q + 2], acc[4 * q + 3]));
            }
        }
    };
    int item = sub * (kT / 64) + wave;
    fetch(item, b0);
#pragma unroll 1
    for (; item < a.nitems; item += 2 * stride) {
        fetch(item + stride, b1);
        compute(item, b0);
        if (item + stride >= a.nitems) break;
        fetch(item + 2 * stride, b0);
        compute(item + stride, b1);
    }
}

// ---- data gradient -------------------------------------------------------------------------------------
// NKS = Cout / 16 reduction steps per tap, GCI input-channel blocks per workgroup (they share the dy
// fragments).  LDS: fragment (g, tap, ks) at ((g * 8 + tap) * NKS + ks) KB; lane l holds
// u[tap][32 (cg GCI + g) + l % 32][16 ks + 8 (l/32) + j] - 16 contiguous bytes of u.
template <int NKS, int GCI>
__global__ __launch_bounds__(kT) void upconv_dgrad_mfma_kernel(UpArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int cg = blockIdx.x % a.nblk, sub = blockIdx.x / a.nblk;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int COUT = 16 * NKS;
    const int m = lane & 31, kh = lane >> 5;
    for (int e = tid; e < GCI * 8 * NKS * 64; e += kT) {
        const int l = e & 63, f = e >> 6;
        const int ks = f % NKS, tap = (f / NKS) & 7, g = f / (8 * NKS);
        const int ci = C * (cg * GCI + g) + (l & 31);
        *reinterpret_cast<uint4 *>(lds + e * 16) = *reinterpret_cast<const uint4 *>(
            a.u + (static_cast<size_t>(tap) * a.cin + ci) * COUT + 16 * ks + 8 * (l >> 5));
    }
    __syncthreads();

#pragma unroll 1
    for (int item = sub * (kT / 64) + wave; item < a.nitems; item += a.wpb * (kT / 64)) {
        const Item o = decode_item(item, a);
        const int w = o.w0 + m;
        const bool ok = w < a.gc.tw;
        const int wl = ok ? w : a.gc.tw - 1;
        f32x16 acc[GCI];
#pragma unroll
        for (int g = 0; g < GCI; ++g)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[g][i] = 0.f;
        // taps in pairs: the dy fragments of the next tap are in flight while the current one is multiplied
        bf16x8 b0[NKS], b1[NKS];
        auto fetch = [&](int tap, bf16x8 (&b)[NKS]) {
            const uint16_t *pdy = a.in + pvox(a.gf, o.tile, 2 * o.d + (tap >> 2), 2 * o.h + ((tap >> 1) & 1),
                                              2 * wl + (tap & 1)) * COUT + 8 * kh;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) b[ks] = *reinterpret_cast<const bf16x8 *>(pdy + 16 * ks);
        };
        auto compute = [&](int tap, const bf16x8 (&b)[NKS]) {
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                for (int g = 0; g < GCI; ++g) {
                    const bf16x8 af = *reinterpret_cast<const bf16x8 *>(
                        lds + ((g * 8 + tap) * NKS + ks) * 1024 + lane * 16);
                    acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b[ks], acc[g], 0, 0, 0);
                }
        };
        fetch(0, b0);
#pragma unroll 1
        for (int tap = 0; tap < 8; tap += 2) {
            fetch(tap + 1, b1);
            compute(tap, b0);
            if (tap + 2 < 8) fetch(tap + 2, b0);
            compute(tap + 1, b1);
        }
        if (ok) {
            uint16_t *px = a.out + pvox(a.gc, o.tile, o.d, o.h, w) * a.cin + C * cg * GCI + 4 * kh;
#pragma unroll
            for (int g = 0; g < GCI; ++g)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2 *>(px + C * g + 8 * q) =
                        make_uint2(pack2(acc[g][4 * q], acc[g][4 * q + 1]), pack2(acc[g][4 * q + 2], acc[g][4 * q + 3]));
        }
    }
}

int dgrad_gci(int cin, int cout) {
    int g = 4;
    while (g > 1 && (g * 8 * (cout / 16) > kMaxFragKB || (cin / C) % g != 0)) g >>= 1;
    return g;
}

int plan(const Geo &gc, int nblk, UpArgs *a) {
    a->nblk = nblk;
    a->nseg = (gc.tw + SEG - 1) / SEG;
    const long long items = 1LL * gc.ntiles * gc.td * gc.th * a->nseg;
    if (items > 0x7fff0000LL) return SP_EGEOM;
    a->nitems = static_cast<int>(items);
    int wpb = kGroups / nblk;
    if (wpb < 1) wpb = 1;
    const long long need = (items + kT / 64 - 1) / (kT / 64);      // workgroups that would each get one pass
    if (wpb > need) wpb = static_cast<int>(need);
    a->wpb = wpb;
    return SP_OK;
}

template <typename K>
int launch(K kernel, const UpArgs &a, int lds_bytes, hipStream_t s) {
    // more than 64 KB of dynamic LDS has to be requested explicitly (cheap; repeated per launch so that
    // every instantiation is covered)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return record_hip(e);
    hipLaunchKernelGGL(kernel, dim3(a.nblk * a.wpb), dim3(kT), lds_bytes, s, a);
    return record_hip(hipGetLastError());
}

}  // namespace

bool upconv_mfma_supported(const Geo &gf, const Geo &gc, int cin, int cout, sp_dtype_t dt) {
    if (dt != SP_BF16 || cin % C != 0 || cout % C != 0 || cin > 256 || cout > 256) return false;
    // element offsets of a voxel inside the tensors stay far below 2^63; segment counts are checked in plan()
    return 1LL * gc.ntiles * gc.td * gc.th * ((gc.tw + SEG - 1) / SEG) <= 0x7fff0000LL;
}

int launch_upconv_fwd_mfma(const void *Px, const void *u, const float *bias, void *Py, const Geo &gf, const Geo &gc,
                           int cin, int cout, hipStream_t s) {
    UpArgs a;
    a.in = static_cast<const uint16_t *>(Px);
    a.u = static_cast<const uint16_t *>(u);
    a.bias = bias;
    a.out = static_cast<uint16_t *>(Py);
    a.gf = gf; a.gc = gc; a.cin = cin; a.cout = cout;
    int rc = plan(gc, cout / C, &a);
    if (rc != SP_OK) return rc;
    const int lds_bytes = 8 * (cin / 16) * 1024;
    switch (cin / C) {
    case 1: return launch(upconv_fwd_mfma_kernel<2>, a, lds_bytes, s);
    case 2: return launch(upconv_fwd_mfma_kernel<4>, a, lds_bytes, s);
    case 3: return launch(upconv_fwd_mfma_kernel<6>, a, lds_bytes, s);
    case 4: return launch(upconv_fwd_mfma_kernel<8>, a, lds_bytes, s);
    case 5: return launch(upconv_fwd_mfma_kernel<10>, a, lds_bytes, s);
    case 6: return launch(upconv_fwd_mfma_kernel<12>, a, lds_bytes, s);
    case 7: return launch(upconv_fwd_mfma_kernel<14>, a, lds_bytes, s);
    case 8: return launch(upconv_fwd_mfma_kernel<16>, a, lds_bytes, s);
    default: return SP_EUNSUPPORTED;
    }
}

int launch_upconv_dgrad_mfma(const void *Pdy, const void *u, void *Pdx, const Geo &gf, const Geo &gc, int cin,
                             int cout, hipStream_t s) {
    UpArgs a;
    a.in = static_cast<const uint16_t *>(Pdy);
    a.u = static_cast<const uint16_t *>(u);
    a.bias = nullptr;
    a.out = static_cast<uint16_t *>(Pdx);
    a.gf = gf; a.gc = gc; a.cin = cin; a.cout = cout;
    const int gci = dgrad_gci(cin, cout);
    int rc = plan(gc, cin / C / gci, &a);
    if (rc != SP_OK) return rc;
    const int nks = cout / 16;
    const int lds_bytes = gci * 8 * nks * 1024;
#define SP3D_DG(NKS)                                                                       \
    case NKS:                                                                              \
        if (gci == 4) return launch(upconv_dgrad_mfma_kernel<NKS, 4>, a, lds_bytes, s);    \
        if (gci == 2) return launch(upconv_dgrad_mfma_kernel<NKS, 2>, a, lds_bytes, s);    \
        return launch(upconv_dgrad_mfma_kernel<NKS, 1>, a, lds_bytes, s);
    switch (nks) {
        SP3D_DG(2) SP3D_DG(4) SP3D_DG(6) SP3D_DG(8) SP3D_DG(10) SP3D_DG(12) SP3D_DG(14) SP3D_DG(16)
    default: return SP_EUNSUPPORTED;
    }
#undef SP3D_DG
}

}  // namespace sp3d
