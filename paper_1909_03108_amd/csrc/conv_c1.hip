// First-layer kernels: 3x3x3 convolution with ONE input channel (the CT volume itself) and a
// multiple of 32 output channels, bf16.  With K = 27 taps the layer is bandwidth-bound (2 bytes in,
// 64 bytes out per voxel at 32 output channels); the matrix cores are used only because they make
// the arithmetic free: the 27 taps, padded to 32, are the GEMM K (forward) or M (weight gradient)
// dimension of a v_mfma_f32_32x32x16_bf16.
//
// Both kernels work on bricks of 4 (D) x 8 (H) x 32 (W) output voxels: the 6 x 10 x 34 input voxels
// around a brick (4 KB) are staged in LDS and every wave owns one plane of the brick.
#include "common.h"

namespace sp3d {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BD = 4, BH = 8, BW = 32;                // brick of output voxels
constexpr int XD = BD + 2, XH = BH + 2, XW = BW + 2;  // input voxels around it
constexpr int XVOX = XD * XH * XW;                    // 2040
constexpr int XLOADS = (XVOX + kThreads - 1) / kThreads;   // 8

struct C1Args {
    const uint16_t *x;     // padded tiles, 1 channel
    const uint16_t *w;     // [27][1][cout]
    const float *bias;
    uint16_t *y;           // forward: padded tiles, cout channels
    const uint16_t *dz;    // weight gradient: padded tiles, cout channels
    float *part;           // weight gradient: [ngroups][cout/32][32 taps][32]
    Geo g;
    int cout;
    int nd, nh, nw;        // bricks per tile
    int nbricks, ngroups;
    int relu;
};

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    union { bf16x2 v; uint32_t u; } r;
    r.v = __builtin_convertvector(f32x2{a, b}, bf16x2);
    return r.u;
}

// element offset inside the staged input brick of tap t relative to an output voxel (0 for the padding taps)
__device__ __forceinline__ int tap_off(int t) {
    return t < 27 ? ((t / 9) * XH + (t / 3) % 3) * XW + t % 3 : 0;
}

// Stage the input voxels around brick (tile, d0, h0, w0) (interior coordinates).  Positions beyond the
// interior and the one voxel around it (ragged bricks) are staged as zero.
__device__ __forceinline__ void stage_x(const C1Args &a, uint16_t *lx, int tile, int d0, int h0, int w0) {
    const Geo &g = a.g;
    const uint16_t *tx = a.x + static_cast<size_t>(tile) * g.tile_vox;
#pragma unroll
    for (int i = 0; i < XLOADS; ++i) {
        const int e = threadIdx.x + i * kThreads;
        if (e < XVOX) {
            const int pd = e / (XH * XW), r = e % (XH * XW), ph = r / XW, pc = r % XW;
            const bool ok = d0 + pd < g.td + 2 && h0 + ph < g.th + 2 && w0 + pc < g.tw + 2;
            lx[e] = ok ? tx[(static_cast<size_t>(d0 + pd) * g.ph + h0 + ph) * g.pw + w0 + pc] : uint16_t(0);
        }
    }
}

// ---- forward ------------------------------------------------------------------------------------------
// D[co][voxel] = sum_tap W[co][tap] * X[tap][voxel]: A = weights (lane: channel lane%32, taps 8*(lane/32)+e of
// each 16-tap half), B = gathered input (lane: voxel lane%32 of a row, the same taps).
__global__ __launch_bounds__(kThreads) void conv_c1_fwd_kernel(C1Args a) {
    __shared__ __attribute__((aligned(16))) uint16_t lx[XVOX + 8];
    const Geo &g = a.g;
    int t = blockIdx.x;
    const int bw_i = t % a.nw; t /= a.nw;
    const int bh_i = t % a.nh; t /= a.nh;
    const int bd_i = t % a.nd; t /= a.nd;
    const int tile = t;
    const int d0 = bd_i * BD, h0 = bh_i * BH, w0 = bw_i * BW;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, hi = lane >> 5;
    stage_x(a, lx, tile, d0, h0, w0);
    int off[2][8];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int e = 0; e < 8; ++e) off[half][e] = tap_off(16 * half + 8 * hi + e);
    __syncthreads();
    const int od = d0 + wave;                         // this wave's output plane
    if (od >= g.td) return;
    uint16_t *ty = a.y + static_cast<size_t>(tile) * g.tile_vox * a.cout;
    for (int cb = 0; cb < a.cout / 32; ++cb) {
        union { bf16x8 v; uint16_t u[8]; } wf[2];
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int tap = 16 * half + 8 * hi + e;
                wf[half].u[e] = tap < 27 ? a.w[tap * a.cout + 32 * cb + col] : uint16_t(0);
            }
        float bv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) bv[i] = a.bias ? a.bias[32 * cb + 8 * (i >> 2) + 4 * hi + (i & 3)] : 0.f;
        for (int r = 0; r < BH; ++r) {
            const int base = (wave * XH + r) * XW + col;
            union { bf16x8 v; uint16_t u[8]; } xf[2];
#pragma unroll
            for (int half = 0; half < 2; ++half)
#pragma unroll
                for (int e = 0; e < 8; ++e) xf[half].u[e] = lx[base + off[half][e]];
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = bv[i];
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[0].v, xf[0].v, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1].v, xf[1].v, acc, 0, 0, 0);
            const int oh = h0 + r, ow = w0 + col;
            if (oh < g.th && ow < g.tw) {
                uint16_t *o = ty + ((static_cast<size_t>(od + 1) * g.ph + oh + 1) * g.pw + ow + 1) * a.cout + 32 * cb + 4 * hi;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float v0 = acc[4 * q], v1 = acc[4 * q + 1], v2 = acc[4 * q + 2], v3 = acc[4 * q + 3];
                    if (a.relu) {
                        v0 = v0 < 0.f ? 0.f : v0; v1 = v1 < 0.f ? 0.f : v1;
                        v2 = v2 < 0.f ? 0.f : v2; v3 = v3 < 0.f ? 0.f : v3;
                    }
                    *reinterpret_cast<uint2 *>(o + 8 * q) = make_uint2(pack2(v0, v1), pack2(v2, v3));
                }
            }
        }
    }
}

// ---- weight (and bias) gradient --------------------------------------------------------------------------
// D[tap][co] = sum_voxels X[tap][voxel] * dz[voxel][co]: A = gathered input (lane: tap lane%32, 8 consecutive
// voxels along W), B = dz read from LDS with the transposing load (lane: channel lane%32, the same 8 voxels).
// The padding row tap 27 of A is the constant 1, so row 27 of D is the bias gradient.
constexpr int ZVOX = BD * BH * BW;                    // 1024 voxels of dz per brick
constexpr int Z_HALF = ZVOX * 32 + 64;                // per 16-channel half: 32-byte voxel records (+ bank offset)
constexpr int WG_LDS = (XVOX + 8) * 2 + 2 * Z_HALF;   // 69760 bytes

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
__device__ __forceinline__ s16x4 tr_read(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(__attribute__((address_space(3))) char *)(p));
}

__global__ __launch_bounds__(kThreads, 2) void wgrad_c1_kernel(C1Args a, int cb) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    uint16_t *lx = reinterpret_cast<uint16_t *>(lds);
    char *lz = lds + (XVOX + 8) * 2;
    const Geo &g = a.g;
    const int group = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, kg = lane >> 5;          // A: tap m, voxels 8*kg .. +7 of a 16-voxel step
    const int toff = tap_off(m);
    // B (transposing read): lane = 16*G + a + 4*j reads voxel 8*(G/2) + j (+4), channel quad a of half G%2
    const int G = lane >> 4, p = lane & 15;
    const char *zlane = lz + (G & 1) * Z_HALF + (8 * (G >> 1) + (p >> 2)) * 32 + (p & 3) * 8;
    const int c4 = threadIdx.x & 3;                   // staging: 16-byte chunk of the 32-channel block
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;

    for (int brick = group; brick < a.nbricks; brick += a.ngroups) {
        int t = brick;
        const int bw_i = t % a.nw; t /= a.nw;
        const int bh_i = t % a.nh; t /= a.nh;
        const int bd_i = t % a.nd; t /= a.nd;
        const int tile = t;
        const int d0 = bd_i * BD, h0 = bh_i * BH, w0 = bw_i * BW;
        __syncthreads();                              // the previous brick's readers are done
        stage_x(a, lx, tile, d0, h0, w0);
        const uint16_t *tz = a.dz + static_cast<size_t>(tile) * g.tile_vox * a.cout + 32 * cb + 8 * c4;
#pragma unroll
        for (int i = 0; i < ZVOX * 4 / kThreads; ++i) {
            const int v = (threadIdx.x + i * kThreads) >> 2;            // brick-local voxel
            const int vd = v / (BH * BW), vh = (v / BW) % BH, vw = v % BW;
            const bool ok = d0 + vd < g.td && h0 + vh < g.th && w0 + vw < g.tw;     // tile interior only
            uint4 q = make_uint4(0, 0, 0, 0);
            if (ok)
                q = *reinterpret_cast<const uint4 *>(
                    tz + ((static_cast<size_t>(d0 + vd + 1) * g.ph + h0 + vh + 1) * g.pw + w0 + vw + 1) * a.cout);
            *reinterpret_cast<uint4 *>(lz + (c4 >> 1) * Z_HALF + v * 32 + (c4 & 1) * 16) = q;
        }
        __syncthreads();
        for (int r = 0; r < BH; ++r)
#pragma unroll
            for (int step = 0; step < 2; ++step) {
                union { bf16x8 v; uint16_t u[8]; } xf;
                const int xb = (wave * XH + r) * XW + 16 * step + 8 * kg + toff;
#pragma unroll
                for (int e = 0; e < 8; ++e) xf.u[e] = m < 27 ? lx[xb + e] : (m == 27 ? uint16_t(0x3F80) : uint16_t(0));
                union { struct { s16x4 lo, hi; } s; bf16x8 v; } zf;
                const char *zp = zlane + ((wave * BH + r) * BW + 16 * step) * 32;
                zf.s.lo = tr_read(zp);
                zf.s.hi = tr_read(zp + 4 * 32);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf.v, zf.v, acc, 0, 0, 0);
            }
    }
    // combine the four waves in a fixed order and write this workgroup's partial [32 taps][32 channels]
    __syncthreads();
    float *red = reinterpret_cast<float *>(lds);
#pragma unroll
    for (int i = 0; i < 16; ++i) red[(wave * 16 + i) * 64 + lane] = acc[i];
    __syncthreads();
    if (wave == 0) {
        float *out = a.part + (static_cast<size_t>(group) * (a.cout / 32) + cb) * 1024;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float s = ((red[i * 64 + lane] + red[(16 + i) * 64 + lane]) + red[(32 + i) * 64 + lane]) +
                            red[(48 + i) * 64 + lane];
            out[(8 * (i >> 2) + 4 * kg + (i & 3)) * 32 + m] = s;      // D row = tap, column = channel
        }
    }
}

// dw[tap][0][co] (tap < 27) and db[co] (row 27) = sum over workgroups, in order, of their partials
__global__ __launch_bounds__(256) void reduce_c1_kernel(const float *__restrict__ part, float *__restrict__ dw,
                                                        float *__restrict__ db, int cout, int ngroups) {
    const int e = blockIdx.x * 256 + threadIdx.x;     // over 28 * cout
    if (e >= 28 * cout) return;
    const int tap = e / cout, co = e % cout;
    const float *p = part + (static_cast<size_t>(co / 32) * 32 + tap) * 32 + co % 32;
    const size_t stride = static_cast<size_t>(cout / 32) * 1024;
    float s = 0.f;
    for (int k = 0; k < ngroups; ++k) s += p[k * stride];
    if (tap < 27) dw[tap * cout + co] = s;
    else if (db) db[co] = s;
}

void plan(const Geo &g, C1Args *a) {
    a->nd = (g.td + BD - 1) / BD;
    a->nh = (g.th + BH - 1) / BH;
    a->nw = (g.tw + BW - 1) / BW;
    const long long nb = 1LL * g.ntiles * a->nd * a->nh * a->nw;
    a->nbricks = static_cast<int>(nb);
    a->ngroups = static_cast<int>(nb < 512 ? nb : 512);
}

}  // namespace

bool conv_c1_supported(const Geo &g, int cin, int cout, sp_dtype_t dt) {
    return dt == SP_BF16 && cin == 1 && cout % 32 == 0 && cout <= 1024 &&
           1LL * g.ntiles * ((g.td + BD - 1) / BD) * ((g.th + BH - 1) / BH) * ((g.tw + BW - 1) / BW) < 0x7fffffffLL;
}

int launch_conv_c1_fwd(const void *Px, const void *w, const float *bias, void *Py, const Geo &g, int cout,
                       bool relu, hipStream_t s) {
    C1Args a{};
    a.x = static_cast<const uint16_t *>(Px);
    a.w = static_cast<const uint16_t *>(w);
    a.bias = bias;
    a.y = static_cast<uint16_t *>(Py);
    a.g = g;
    a.cout = cout;
    a.relu = relu ? 1 : 0;
    plan(g, &a);
    hipLaunchKernelGGL(conv_c1_fwd_kernel, dim3(a.nbricks), dim3(kThreads), 0, s, a);
    return record_hip(hipGetLastError());
}

size_t wgrad_c1_ws_bytes(const Geo &g, int cout) {
    C1Args a{};
    plan(g, &a);
    return static_cast<size_t>(a.ngroups) * (cout / 32) * 1024 * sizeof(float);
}

int launch_wgrad_c1(const void *Px, const void *Pdz, float *dw, float *db, const Geo &g, int cout, void *ws,
                    hipStream_t s) {
    C1Args a{};
    a.x = static_cast<const uint16_t *>(Px);
    a.dz = static_cast<const uint16_t *>(Pdz);
    a.part = static_cast<float *>(ws);
    a.g = g;
    a.cout = cout;
    plan(g, &a);
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(wgrad_c1_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS);
    if (attr != hipSuccess) return record_hip(attr);
    for (int cb = 0; cb < cout / 32; ++cb)
        hipLaunchKernelGGL(wgrad_c1_kernel, dim3(a.ngroups), dim3(kThreads), WG_LDS, s, a, cb);
    int rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    hipLaunchKernelGGL(reduce_c1_kernel, dim3((28 * cout + 255) / 256), dim3(256), 0, s, a.part, dw, db, cout,
                       a.ngroups);
    return record_hip(hipGetLastError());
}

}  // namespace sp3d
