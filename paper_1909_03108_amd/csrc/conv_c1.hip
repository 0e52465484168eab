// First-layer kernels: 3x3x3 convolution with ONE input channel (the CT volume itself) and a
// multiple of 32 output channels, bf16.  With K = 27 taps the layer is bandwidth-bound (2 bytes in,
// 64 bytes out per voxel at 32 output channels); the matrix cores are used only because they make
// the arithmetic free: the 27 taps, padded to 32, are the GEMM K (forward) or M (weight gradient)
// dimension of a v_mfma_f32_32x32x16_bf16.
//
// Both kernels stage the input voxels around a brick of output voxels in LDS (2-byte elements, gathered per
// tap): the weight gradient works on bricks of 4 (D) x 8 (H) x 32 (W) with one plane per wave, the forward pass
// on bricks of 1 x 32 x 32 with 8 rows per wave.
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
    uint16_t *bits;        // forward, optional: one-bit ReLU mask of y (layout: sp3d.h, sp_relu_bits)
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

// ReLU on two packed bf16 values: a bf16 with its sign bit set is a negative 16-bit integer, so the signed
// integer maximum with 0 clears exactly the negative values (and -0); one v_pk_max_i16 per pair
__device__ __forceinline__ uint32_t relu2(uint32_t p) {
    typedef short s16x2 __attribute__((ext_vector_type(2)));
    union { uint32_t u; s16x2 v; } a, r;
    a.u = p;
    r.v = __builtin_elementwise_max(a.v, s16x2{0, 0});
    return r.u;
}

// element offset inside the staged input brick of tap t relative to an output voxel (0 for the padding taps)
__host__ __device__ constexpr int tap_off(int t) {
    return t < 27 ? ((t / 9) * XH + (t / 3) % 3) * XW + t % 3 : 0;
}

// ---- forward ------------------------------------------------------------------------------------------
// D[co][voxel] = sum_tap W[co][tap] * X[tap][voxel]: A = weights (lane: channel lane%32, taps 8*(lane/32)+e of
// each 16-tap half), B = gathered input (lane: voxel lane%32 of a row, the same taps).
// The kernel is bound by its 64 bytes of output per voxel, so the stores are shaped for the memory system: a
// finished row (32 voxels x 64 bytes) goes through a wave-private LDS buffer, in which lane (voxel, half) writes
// its four 8-byte pieces and from which lane l reads the 16 contiguous bytes l % 4 of voxel l / 4, so that one
// store instruction writes 1 KB of consecutive memory (sixteen whole voxel records) instead of 8-byte pieces
// 64 bytes apart.  Two rows are in flight at a time so that the second row's MFMAs cover the first row's epilogue.
constexpr int YROW = 72;                              // LDS bytes per voxel record: 64 + 8 of padding (8-byte writes
                                                      // 72 bytes apart fall into 32 different bank pairs)
constexpr int YBUF = 32 * YROW;                       // one row
// Forward bricks are one plane thick: 32 rows (8 per wave) x 32 voxels along W, so that a workgroup writes a
// compact block of adjacent rows while it walks along W (with bricks four planes thick the same stores ran
// slower: the four waves then wrote into planes megabytes apart).
constexpr int FH = 32, FXD = 3, FXH = FH + 2;         // brick rows; input planes and rows around a brick
constexpr int FXROWS = FXD * FXH;                     // 102 staged rows of XW voxels
constexpr int FXVOX = FXROWS * XW;                    // 3468
constexpr int FRW = (FXROWS + 3) / 4;                 // rows per wave when staging: 26

__host__ __device__ constexpr int fwd_tap_off(int t) {
    return t < 27 ? ((t / 9) * FXH + (t / 3) % 3) * XW + t % 3 : 0;
}

// A workgroup walks along W over the bricks of one (tile, plane, group of 32 rows): while it computes a brick,
// the input voxels of the next one are already on their way into registers (wave w fetches rows w, w + 4, ...;
// lanes 0..33 one voxel each), and they are written to the other half of a double-buffered LDS array afterwards,
// so neither the memory latency nor more than one barrier per brick lies on the critical path.
// BITS: the kernel also writes the one-bit form of its result's ReLU mask.  The matrix cores hand lane (voxel,
// half) the channels 8 q + 4 half + i of its voxel, which is the order of the bits in the mask's 16-bit words:
// each lane collects its word from the packed results and stores it (a wave: 128 consecutive bytes per block).
template <bool RELU, bool HAS_BIAS, bool BITS>
__global__ __launch_bounds__(kThreads) void conv_c1_fwd_kernel(C1Args a, int nhg) {
    __shared__ __attribute__((aligned(16))) uint16_t lx[2][FXVOX + 8];
    __shared__ __attribute__((aligned(16))) char ly[kThreads / 64][2][YBUF];
    const Geo &g = a.g;
    // workgroup ids go round the 8 XCDs; renumbered, an XCD holds a run of neighbouring row blocks and planes
    int t = (gridDim.x & 7) == 0 ? (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    const int bh_i = t % nhg; t /= nhg;
    const int od = t % g.td; t /= g.td;               // output plane (interior coordinate)
    const int tile = t;
    const int h0 = bh_i * FH;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, hi = lane >> 5;
    const uint16_t *tx = a.x + static_cast<size_t>(tile) * g.tile_vox;
    uint16_t *ty = a.y + static_cast<size_t>(tile) * g.tile_vox * a.cout;

    // staging: element offsets of this lane's voxel in each of its rows (-1: beyond the interior and the one
    // voxel around it, staged as zero); the W position advances by BW per brick
    int xsrc[FRW];
#pragma unroll
    for (int i = 0; i < FRW; ++i) {
        const int row = wave + 4 * i, pd = row / FXH, ph = row % FXH;
        const bool ok = row < FXROWS && lane < XW && h0 + ph < g.th + 2;
        xsrc[i] = ok ? ((od + pd) * g.ph + h0 + ph) * g.pw + lane : -1;
    }
    uint16_t xr[FRW];
    auto fetch = [&](int w0) {
#pragma unroll
        for (int i = 0; i < FRW; ++i) {
            const bool ok = xsrc[i] >= 0 && w0 + lane < g.tw + 2;
            xr[i] = ok ? tx[xsrc[i] + w0] : uint16_t(0);
        }
    };
    auto commit = [&](uint16_t *dst) {
#pragma unroll
        for (int i = 0; i < FRW; ++i)
            if (wave + 4 * i < FXROWS && lane < XW) dst[(wave + 4 * i) * XW + lane] = xr[i];
    };
    fetch(0);
    commit(lx[0]);

    int off[2][8];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int e = 0; e < 8; ++e) off[half][e] = hi ? fwd_tap_off(16 * half + 8 + e) : fwd_tap_off(16 * half + e);
    const int r0 = wave * (FH / 4);                   // this wave's rows of the brick: r0 .. r0 + 7
    const bool rows_ok = h0 + r0 < g.th;
    char *wy = &ly[wave][0][0];
    char *wr_at = wy + col * YROW + 8 * hi;           // this lane's pieces: + 16 q
    const int rv = lane >> 2, rp = lane & 3;          // read back: voxel rv (+16), 16-byte piece rp
    const char *rd_at = wy + rv * YROW + 16 * rp;
    // weights and bias of the (first) output block; wider layers reload them per block inside the loop
    const int ncb = a.cout / 32;
    union WF { bf16x8 v; uint16_t u[8]; };
    WF wf[2];
    f32x16 bv;
    auto load_weights = [&](int cb) {
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int tap = 16 * half + 8 * hi + e;
                wf[half].u[e] = tap < 27 ? a.w[tap * a.cout + 32 * cb + col] : uint16_t(0);
            }
#pragma unroll
        for (int i = 0; i < 16; ++i) bv[i] = HAS_BIAS ? a.bias[32 * cb + 8 * (i >> 2) + 4 * hi + (i & 3)] : 0.f;
    };
    load_weights(0);
    __syncthreads();

    for (int bw_i = 0; bw_i < a.nw; ++bw_i) {
        const int w0 = bw_i * BW;
        const uint16_t *cur = lx[bw_i & 1];
        if (bw_i + 1 < a.nw) fetch(w0 + BW);
        if (rows_ok) {
            for (int cb = 0; cb < ncb; ++cb) {
                if (ncb > 1) load_weights(cb);
#pragma unroll 1
                for (int r = 0; r < FH / 4; r += 2) {
                    WF xf[2][2];
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const int base = (r0 + r + k) * XW + col;
#pragma unroll
                        for (int half = 0; half < 2; ++half)
#pragma unroll
                            for (int e = 0; e < 8; ++e) xf[k][half].u[e] = cur[base + off[half][e]];
                    }
                    f32x16 acc[2];
#pragma unroll
                    for (int k = 0; k < 2; ++k)
                        acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[0].v, xf[k][0].v, bv, 0, 0, 0);
#pragma unroll
                    for (int k = 0; k < 2; ++k)
                        acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1].v, xf[k][1].v, acc[k], 0, 0, 0);
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        uint32_t word = 0;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            uint32_t p0 = pack2(acc[k][4 * q], acc[k][4 * q + 1]), p1 = pack2(acc[k][4 * q + 2], acc[k][4 * q + 3]);
                            if (RELU) { p0 = relu2(p0); p1 = relu2(p1); }
                            *reinterpret_cast<uint2 *>(wr_at + k * YBUF + 16 * q) = make_uint2(p0, p1);
                            if (BITS)       // positive: not zero, not negative, not NaN
                                word |= (((p0 & 0xffffu) - 1u < 0x7f80u ? 1u : 0u) | ((p0 >> 16) - 1u < 0x7f80u ? 2u : 0u) |
                                         ((p1 & 0xffffu) - 1u < 0x7f80u ? 4u : 0u) | ((p1 >> 16) - 1u < 0x7f80u ? 8u : 0u))
                                        << (4 * q);
                        }
                        if (BITS) {
                            const int oh = h0 + r0 + r + k;
                            const size_t vox = static_cast<size_t>(tile) * g.tile_vox +
                                               (static_cast<size_t>(od + 1) * g.ph + oh + 1) * g.pw + w0 + 1 + col;
                            if (oh < g.th && w0 + col < g.tw)
                                a.bits[(vox * ncb + cb) * 2 + hi] = static_cast<uint16_t>(word);
                        }
                    }
                    // the LDS unit serves a wave's accesses in order, so the reads below see the writes above
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const int oh = h0 + r0 + r + k;
                        uint16_t *orow = ty + ((static_cast<size_t>(od + 1) * g.ph + oh + 1) * g.pw + w0 + 1) * a.cout +
                                         32 * cb + 8 * rp;
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            const int v = rv + 16 * j;
                            const uint2 lo = *reinterpret_cast<const uint2 *>(rd_at + k * YBUF + 16 * j * YROW);
                            const uint2 hi2 = *reinterpret_cast<const uint2 *>(rd_at + k * YBUF + 16 * j * YROW + 8);
                            if (oh < g.th && w0 + v < g.tw)
                                st_stream16(orow + static_cast<size_t>(v) * a.cout, make_uint4(lo.x, lo.y, hi2.x, hi2.y));
                        }
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                }
            }
        }
        if (bw_i + 1 < a.nw) commit(lx[(bw_i + 1) & 1]);
        __syncthreads();
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

constexpr int XROWS = XD * XH;                        // 60 input rows of XW voxels around a brick
constexpr int XRW = (XROWS + 3) / 4;                  // rows per wave when staging: 15
constexpr int ZLD = ZVOX * 4 / kThreads;              // 16-byte pieces of dz per thread and brick: 16

// The loads of a workgroup's next brick (x: wave w takes rows w, w + 4, ..., lanes 0..33 one voxel each; dz: four
// lanes per voxel, 16 bytes each) are issued before the MFMAs of the current brick and land in registers while
// those run; they go to LDS between two barriers afterwards.
__global__ __launch_bounds__(kThreads, 2) void wgrad_c1_kernel(C1Args a, int cb) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    uint16_t *lx = reinterpret_cast<uint16_t *>(lds);
    char *lz = lds + (XVOX + 8) * 2;
    const Geo &g = a.g;
    const int group = (gridDim.x & 7) == 0 ? (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
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

    uint16_t xr[XRW];
    uint4 zr[ZLD];
    auto fetch = [&](int brick) {
        int t = brick;
        const int bw_i = t % a.nw; t /= a.nw;
        const int bh_i = t % a.nh; t /= a.nh;
        const int bd_i = t % a.nd; t /= a.nd;
        const int tile = t;
        const int d0 = bd_i * BD, h0 = bh_i * BH, w0 = bw_i * BW;
        const uint16_t *tx = a.x + static_cast<size_t>(tile) * g.tile_vox;
#pragma unroll
        for (int i = 0; i < XRW; ++i) {
            const int row = wave + 4 * i, pd = row / XH, ph = row % XH;
            // beyond the interior and the one voxel around it (ragged bricks): zero
            const bool ok = row < XROWS && lane < XW && d0 + pd < g.td + 2 && h0 + ph < g.th + 2 && w0 + lane < g.tw + 2;
            xr[i] = ok ? tx[(static_cast<size_t>(d0 + pd) * g.ph + h0 + ph) * g.pw + w0 + lane] : uint16_t(0);
        }
        const uint16_t *tz = a.dz + static_cast<size_t>(tile) * g.tile_vox * a.cout + 32 * cb + 8 * c4;
#pragma unroll
        for (int i = 0; i < ZLD; ++i) {
            const int v = (threadIdx.x + i * kThreads) >> 2;            // brick-local voxel
            const int vd = v / (BH * BW), vh = (v / BW) % BH, vw = v % BW;
            const bool ok = d0 + vd < g.td && h0 + vh < g.th && w0 + vw < g.tw;     // tile interior only
            zr[i] = make_uint4(0, 0, 0, 0);
            if (ok)
                zr[i] = *reinterpret_cast<const uint4 *>(
                    tz + ((static_cast<size_t>(d0 + vd + 1) * g.ph + h0 + vh + 1) * g.pw + w0 + vw + 1) * a.cout);
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < XRW; ++i)
            if (wave + 4 * i < XROWS && lane < XW) lx[(wave + 4 * i) * XW + lane] = xr[i];
#pragma unroll
        for (int i = 0; i < ZLD; ++i) {
            const int v = (threadIdx.x + i * kThreads) >> 2;
            *reinterpret_cast<uint4 *>(lz + (c4 >> 1) * Z_HALF + v * 32 + (c4 & 1) * 16) = zr[i];
        }
    };

    if (group < a.nbricks) fetch(group);
    for (int brick = group; brick < a.nbricks; brick += a.ngroups) {
        commit();
        __syncthreads();
        if (brick + a.ngroups < a.nbricks) fetch(brick + a.ngroups);
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
        __syncthreads();                              // this brick's readers are done before the next commit
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
    // sixteen loads in flight, added in workgroup order (one dependent load per partial made the 512-step chain
    // of every output cost its full memory latency each time: 126 us for 900 outputs)
    float s = 0.f;
    int k = 0;
    for (; k + 16 <= ngroups; k += 16) {
        float v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = p[(k + i) * stride];
#pragma unroll
        for (int i = 0; i < 16; ++i) s += v[i];
    }
    for (; k < ngroups; ++k) s += p[k * stride];
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
    return !g.flat && dt == SP_BF16 && cin == 1 && cout % 32 == 0 && cout <= 1024 &&
           1LL * g.ntiles * g.td * ((g.th + BH - 1) / BH) * ((g.tw + BW - 1) / BW) < 0x7fffffffLL;
}

int launch_conv_c1_fwd(const void *Px, const void *w, const float *bias, void *Py, const Geo &g, int cout,
                       bool relu, hipStream_t s, void *bits) {
    if (bits && !relu) return SP_EINVAL;
    C1Args a{};
    a.x = static_cast<const uint16_t *>(Px);
    a.w = static_cast<const uint16_t *>(w);
    a.bias = bias;
    a.y = static_cast<uint16_t *>(Py);
    a.bits = static_cast<uint16_t *>(bits);
    a.g = g;
    a.cout = cout;
    a.relu = relu ? 1 : 0;
    plan(g, &a);
    const int nhg = (g.th + FH - 1) / FH;
    const dim3 grid(static_cast<unsigned>(1LL * g.ntiles * g.td * nhg)), block(kThreads);
    if (bits) {
        if (bias) hipLaunchKernelGGL((conv_c1_fwd_kernel<true, true, true>), grid, block, 0, s, a, nhg);
        else hipLaunchKernelGGL((conv_c1_fwd_kernel<true, false, true>), grid, block, 0, s, a, nhg);
    } else if (relu) {
        if (bias) hipLaunchKernelGGL((conv_c1_fwd_kernel<true, true, false>), grid, block, 0, s, a, nhg);
        else hipLaunchKernelGGL((conv_c1_fwd_kernel<true, false, false>), grid, block, 0, s, a, nhg);
    } else {
        if (bias) hipLaunchKernelGGL((conv_c1_fwd_kernel<false, true, false>), grid, block, 0, s, a, nhg);
        else hipLaunchKernelGGL((conv_c1_fwd_kernel<false, false, false>), grid, block, 0, s, a, nhg);
    }
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
