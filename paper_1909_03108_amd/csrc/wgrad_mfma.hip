// bf16 weight gradient of the 3x3x3 convolution for channel counts that are multiples of 32 on the
// gfx950 matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulation), plus the bias gradient.
// The kernel proper handles one (32 input channels) x (32 output channels) pair; wider layers give
// every pair its own set of workgroups in the same launch (the pairs are independent).
//
//   dw[tap][ci][co] = sum over tiles and interior voxels v of  Px[v + tap][ci] * Pdz[v + (1,1,1)][co]
//
// GEMM view: M = ci, N = co, K = voxels.  The reduction runs over voxels, but NDHWC keeps channels
// contiguous, so both operands are read from LDS with the transposing load ds_read_b64_tr_b16,
// which hands every lane 4 voxels of one channel.
//
// Work decomposition.  A workgroup (4 waves) walks over work items = (tile, D chunk, 8 x 32 patch).
// For an item it marches along D: x plane D (10 x 34 voxels, with halo) and the dz planes D, D-1,
// D-2 (8 x 32 voxels, zero outside the tile interior) sit in LDS; x plane D meets dz plane D-kd
// through tap kd.  Wave q owns the 16 x 16 quadrant (ci half, co half) of all 27 taps (108
// accumulator registers) for the whole kernel.  Per x row R it reads the three kw-shifted x
// fragments once and the dz fragments of row R for the three planes once; the dz fragments of
// rows R-1, R-2 are still in registers, so 6 fragment reads feed 27 MFMAs.
// Each workgroup writes its partial dw / db to the workspace; a second kernel adds the partials in
// workgroup order, so the result does not depend on scheduling.
#include "common.h"

namespace sp3d {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int C = 32;
constexpr int kThreads = 512;                 // 8 waves: 4 output quadrants x 2 row groups
constexpr int PH = 8, PW = 32;
constexpr int XR = PH + 2, XC = PW + 2;
constexpr int XVOX = XR * XC;                 // 340
constexpr int ZVOX = PH * PW;                 // 256
constexpr int GR = PH / 2;                    // dz rows per row group (4); x rows per group: GR + 2
// LDS: channel halves are separate arrays of 32-byte voxel records; the +64 makes the two halves
// written by neighbouring lanes land in different banks.
constexpr int X_HALF = XVOX * 32 + 64;        // 10944
constexpr int X_BYTES = 2 * X_HALF;           // 21888 per buffer, 2 buffers
constexpr int Z_HALF = ZVOX * 32 + 64;        // 8256
constexpr int Z_PLANE = 2 * Z_HALF;           // 16512 per slot, 4 slots
constexpr int STAGE_BYTES = 2 * X_BYTES + 4 * Z_PLANE;       // 109824
constexpr int RED_BYTES = 4 * 27 * 4 * 64 * 4;               // row-group combine at the end: 110592
constexpr int LDS_BYTES = STAGE_BYTES > RED_BYTES ? STAGE_BYTES : RED_BYTES;
static_assert(kThreads * 8 * 4 <= LDS_BYTES, "bias reduction scratch must fit");
constexpr int kMaxGroups = 256;               // workgroups (= partial results); one per CU

struct WgradArgs {
    const uint16_t *x;
    const uint16_t *dz;
    float *part_w;        // [ngroups][27][32][32]
    float *part_b;        // [ngroups][32]
    Geo g;
    int x_cs, dz_cs;      // channels per voxel of x and dz
    int nco;              // output blocks; pair p = (input chunk p / nco, output block p % nco)
    int gpp;              // workgroups per pair
    int dchunk, nd, nh, nw;
    int nitems;           // work items per pair
    int ngroups;          // real workgroups = pairs * gpp; grid is rounded up to a multiple of 8
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Transposing LDS read of one MFMA operand half: 16 voxels x 16 channels -> 4 voxels per lane.
__device__ __forceinline__ s16x4 tr_read(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4 *)(__attribute__((address_space(3))) char *)(p));
}

// One operand fragment (32 voxels x 16 channels): voxels 0..15 then 16..31 of a row.
__device__ __forceinline__ bf16x8 frag(const char *p) {
    union { struct { s16x4 lo, hi; } s; bf16x8 v; } u;
    u.s.lo = tr_read(p);
    u.s.hi = tr_read(p + 16 * 32);
    return u.v;
}

// x plane D (in xcur) against dz planes D, D-1, D-2 (ring slots (P - kd) mod 4) for the GR dz rows
// of this wave's row group; xlane / zlane already point at the group's first row.
template <int P>   // P = D mod 4
__device__ __forceinline__ void plane_step(const char *xlane, const char *zlane, f32x4 (&acc)[27]) {
    bf16x8 zf[3][3];   // [kd][row mod 3]
#pragma unroll
    for (int R = 0; R < GR + 2; ++R) {
        bf16x8 xf[3];
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) xf[kw] = frag(xlane + (R * XC + kw) * 32);
        if (R < GR) {
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
                zf[kd][R % 3] = frag(zlane + ((P - kd + 4) % 4) * Z_PLANE + R * PW * 32);
        }
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            const int h = R - kh;
            if (h < 0 || h >= GR) continue;
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    const int tap = (kd * 3 + kh) * 3 + kw;
                    acc[tap] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[kw], zf[kd][h % 3], acc[tap],
                                                                       0, 0, 0);
                }
        }
    }
}

__global__ __launch_bounds__(kThreads) void wgrad_mfma_kernel(WgradArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const Geo &g = a.g;
    const int per_xcd = gridDim.x >> 3;
    const int group = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (group >= a.ngroups) return;
    const int pair = group / a.gpp, gsub = group % a.gpp;
    const int x_co = C * (pair / a.nco), dz_co = C * (pair % a.nco);   // channel offsets of this pair
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = (wave >> 1) & 1, qo = wave & 1;   // ci half, co half of this wave's quadrant
    const int kg = wave >> 2;                         // row group: dz rows [GR*kg, GR*kg + GR)
    char *xbuf = lds;
    char *zbuf = lds + 2 * X_BYTES;
    // per-lane part of the transposing-read address: lane = 16*G + a + 4*j reads voxel 4G + j,
    // channel quad a (4 channels = 8 bytes) of its wave's channel half
    const int G = lane >> 4, p = lane & 15;
    const int lane_off = (4 * G + (p >> 2)) * 32 + (p & 3) * 8;
    const char *xlane = xbuf + qi * X_HALF + lane_off + kg * GR * XC * 32;
    const char *zlane = zbuf + qo * Z_HALF + lane_off + kg * GR * PW * 32;

    // Staging slots of this thread (fixed for the whole kernel).  c4 = which 16-byte chunk of the
    // 64-byte voxel record (channels 8*c4..+7).  x plane: rows of 34 voxels = 128 "main" chunks
    // (voxels 0..31) + 8 "edge" chunks (voxels 32, 33); main rows sr + 4i, edge row = tid / 8.
    const int c4 = tid & 3;
    const int sr = tid >> 7, sv = (tid & 127) >> 2;          // main: row group, voxel column
    const int er = tid >> 3, ev = 32 + ((tid & 7) >> 2);     // edge: row, voxel column (tid < 80)
    const int lds_c = (c4 >> 1) * X_HALF + (c4 & 1) * 16;
    const int xdst0 = lds_c + (sr * XC + sv) * 32;           // + 4i rows
    const int xdste = lds_c + (er * XC + ev) * 32;
    const int zdst0 = (c4 >> 1) * Z_HALF + (c4 & 1) * 16 + (sr * PW + sv) * 32;   // + 4i rows

    f32x4 acc[27];
#pragma unroll
    for (int t = 0; t < 27; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    float bsum[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) bsum[j] = 0.f;

    const size_t xplane = static_cast<size_t>(g.ph) * g.pw * a.x_cs, zplane = static_cast<size_t>(g.ph) * g.pw * a.dz_cs;
    const int xrow_elems = g.pw * a.x_cs, zrow_elems = g.pw * a.dz_cs;

    for (int item = gsub; item < a.nitems; item += a.gpp) {
        int t = item;
        const int pw_i = t % a.nw; t /= a.nw;
        const int ph_i = t % a.nh; t /= a.nh;
        const int pd_i = t % a.nd; t /= a.nd;
        const int tile = t;
        const int d0 = pd_i * a.dchunk, h0 = ph_i * PH, w0 = pw_i * PW;
        const int dn = min(a.dchunk, g.td - d0);
        const uint16_t *tx = a.x + static_cast<size_t>(tile) * g.tile_vox * a.x_cs + x_co;
        const uint16_t *tz = a.dz + static_cast<size_t>(tile) * g.tile_vox * a.dz_cs + dz_co;

        // source offsets inside a plane and validity (x: inside the padded tile; dz: tile interior)
        const int xsrc0 = ((h0 + sr) * g.pw + w0 + sv) * a.x_cs + c4 * 8;
        const int xsrce = ((h0 + er) * g.pw + w0 + ev) * a.x_cs + c4 * 8;
        const int zsrc0 = ((h0 + sr + 1) * g.pw + w0 + sv + 1) * a.dz_cs + c4 * 8;
        bool xok[3], zok[2];
#pragma unroll
        for (int i = 0; i < 3; ++i)
            xok[i] = sr + 4 * i < XR && h0 + sr + 4 * i < g.ph && w0 + sv < g.pw;
        const bool eok = tid < 8 * XR && h0 + er < g.ph && w0 + ev < g.pw;
#pragma unroll
        for (int i = 0; i < 2; ++i) zok[i] = h0 + sr + 4 * i < g.th && w0 + sv < g.tw;

        // staged chunks travel in registers from the global loads (issued before a plane's MFMAs)
        // to the LDS writes (after them)
        uint4 xs0, xs1, xs2, xs3, zs0, zs1;
        const uint4 zero4 = make_uint4(0, 0, 0, 0);
#define SP3D_LDG(ok, ptr) ((ok) ? *reinterpret_cast<const uint4 *>(ptr) : zero4)
#define SP3D_FETCH(D)                                                                  \
    do {                                                                               \
        const uint16_t *px = tx + (d0 + (D)) * xplane;                                 \
        xs0 = SP3D_LDG(xok[0], px + xsrc0);                                            \
        xs1 = SP3D_LDG(xok[1], px + xsrc0 + 4 * xrow_elems);                           \
        xs2 = SP3D_LDG(xok[2], px + xsrc0 + 8 * xrow_elems);                           \
        xs3 = SP3D_LDG(eok, px + xsrce);                                               \
        const bool zreal = (D) < dn;                                                   \
        const uint16_t *pz = tz + (d0 + (D) + 1) * zplane;                             \
        zs0 = SP3D_LDG(zreal && zok[0], pz + zsrc0);                                   \
        zs1 = SP3D_LDG(zreal && zok[1], pz + zsrc0 + 4 * zrow_elems);                  \
    } while (0)
#define SP3D_BSUM(V_)                                                                  \
    do {                                                                               \
        bsum[0] += __uint_as_float((V_).x << 16); bsum[1] += __uint_as_float((V_).x & 0xffff0000u); \
        bsum[2] += __uint_as_float((V_).y << 16); bsum[3] += __uint_as_float((V_).y & 0xffff0000u); \
        bsum[4] += __uint_as_float((V_).z << 16); bsum[5] += __uint_as_float((V_).z & 0xffff0000u); \
        bsum[6] += __uint_as_float((V_).w << 16); bsum[7] += __uint_as_float((V_).w & 0xffff0000u); \
    } while (0)
#define SP3D_COMMIT(D)                                                                 \
    do {                                                                               \
        char *xp = xbuf + ((D) & 1) * X_BYTES;                                         \
        *reinterpret_cast<uint4 *>(xp + xdst0) = xs0;                                  \
        *reinterpret_cast<uint4 *>(xp + xdst0 + 4 * XC * 32) = xs1;                    \
        if (sr + 8 < XR) *reinterpret_cast<uint4 *>(xp + xdst0 + 8 * XC * 32) = xs2;   \
        if (tid < 8 * XR) *reinterpret_cast<uint4 *>(xp + xdste) = xs3;                \
        char *zp = zbuf + ((D) & 3) * Z_PLANE;                                         \
        *reinterpret_cast<uint4 *>(zp + zdst0) = zs0;                                  \
        *reinterpret_cast<uint4 *>(zp + zdst0 + 4 * PW * 32) = zs1;                    \
        SP3D_BSUM(zs0);                                                                \
        SP3D_BSUM(zs1);                                                                \
    } while (0)

        // prologue: dz planes -1 and -2 (ring slots 3 and 2) are zero; stage x plane 0 and dz plane 0
        __syncthreads();   // every wave is done reading the previous item's planes
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            *reinterpret_cast<uint4 *>(zbuf + 2 * Z_PLANE + zdst0 + 4 * i * PW * 32) = zero4;
            *reinterpret_cast<uint4 *>(zbuf + 3 * Z_PLANE + zdst0 + 4 * i * PW * 32) = zero4;
        }
        SP3D_FETCH(0);
        SP3D_COMMIT(0);
        __syncthreads();

        // x is double buffered and the dz ring has 4 slots, so plane D+1 can be written while other
        // waves still read planes D, D-1, D-2: one barrier per plane.
        const int nplanes = dn + 2;
        for (int D = 0; D < nplanes; D += 4) {
#pragma unroll
            for (int ph = 0; ph < 4; ++ph) {
                const int Dp = D + ph;
                if (Dp < nplanes) {
                    const bool more = Dp + 1 < nplanes;
                    if (more) SP3D_FETCH(Dp + 1);
                    const char *xl = xlane + (Dp & 1) * X_BYTES;
                    if (ph == 0) plane_step<0>(xl, zlane, acc);
                    else if (ph == 1) plane_step<1>(xl, zlane, acc);
                    else if (ph == 2) plane_step<2>(xl, zlane, acc);
                    else plane_step<3>(xl, zlane, acc);
                    if (more) SP3D_COMMIT(Dp + 1);
                    __syncthreads();
                }
            }
        }
    }

#undef SP3D_LDG
#undef SP3D_FETCH
#undef SP3D_BSUM
#undef SP3D_COMMIT
    // Combine the two row groups in a fixed order (group 0 + group 1) and write this workgroup's
    // partial result.
    __syncthreads();
    float *red = reinterpret_cast<float *>(lds);
    const int quad = wave & 3;
    if (kg == 1) {
#pragma unroll
        for (int t = 0; t < 27; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[((quad * 27 + t) * 4 + i) * 64 + lane] = acc[t][i];
    }
    __syncthreads();
    if (kg == 0) {
        float *pw = a.part_w + static_cast<size_t>(group) * 27 * C * C;
#pragma unroll
        for (int t = 0; t < 27; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                pw[(t * C + 16 * qi + 4 * G + i) * C + 16 * qo + p] =
                    acc[t][i] + red[((quad * 27 + t) * 4 + i) * 64 + lane];
    }
    // bias partial: threads with the same chunk index hold sums of the same 8 channels
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; ++j) red[tid * 8 + j] = bsum[j];
    __syncthreads();
    if (tid < C) {
        const int chunk = tid >> 3, j = tid & 7;
        float s = 0.f;
        for (int k = chunk; k < kThreads; k += 4) s += red[k * 8 + j];
        a.part_b[group * C + tid] = s;
    }
}

void plan(const Geo &g, int cin, int cout, WgradArgs *a) {
    const int npairs = (cin / C) * (cout / C);
    a->x_cs = cin;
    a->dz_cs = cout;
    a->nco = cout / C;
    a->nh = (g.th + PH - 1) / PH;
    a->nw = (g.tw + PW - 1) / PW;
    int gpp = kMaxGroups / npairs;                    // about one workgroup per CU in total
    if (gpp < 1) gpp = 1;
    const long long base = 1LL * g.ntiles * a->nh * a->nw;
    int dchunk = g.td;
    while (base * ((g.td + dchunk - 1) / dchunk) < gpp && dchunk > 16) dchunk = (dchunk + 1) / 2;
    a->dchunk = dchunk;
    a->nd = (g.td + dchunk - 1) / dchunk;
    const long long items = base * a->nd;
    a->nitems = static_cast<int>(items);
    a->gpp = static_cast<int>(items < gpp ? items : gpp);
    a->ngroups = a->gpp * npairs;
}

// dw[tap][ci][co] = sum over the workgroups of pair (ci/32, co/32), in workgroup order, of their partial
// [tap][ci%32][co%32]; db[co] likewise from the pairs of input chunk 0.
__global__ __launch_bounds__(256) void reduce_wgrad_kernel(const float *__restrict__ part_w,
                                                           const float *__restrict__ part_b,
                                                           float *__restrict__ dw, float *__restrict__ db,
                                                           int cin, int cout, int gpp) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    const int nw_ = 27 * cin * cout;
    if (e < nw_) {
        const int co = e % cout, ci = (e / cout) % cin, tap = e / (cout * cin);
        const int pair = (ci / C) * (cout / C) + co / C;
        const float *p = part_w + (static_cast<size_t>(pair) * gpp * 27 + tap) * C * C + (ci % C) * C + co % C;
        float s = 0.f;
        int k = 0;
        for (; k + 4 <= gpp; k += 4) {          // loads issued together, additions kept in order
            const float p0 = p[static_cast<size_t>(k) * 27 * C * C], p1 = p[static_cast<size_t>(k + 1) * 27 * C * C];
            const float p2 = p[static_cast<size_t>(k + 2) * 27 * C * C], p3 = p[static_cast<size_t>(k + 3) * 27 * C * C];
            s = (((s + p0) + p1) + p2) + p3;
        }
        for (; k < gpp; ++k) s += p[static_cast<size_t>(k) * 27 * C * C];
        dw[e] = s;
    } else if (db && e < nw_ + cout) {
        const int co = e - nw_;
        const float *p = part_b + static_cast<size_t>(co / C) * gpp * C + co % C;     // pairs (0, co/32)
        float s = 0.f;
        for (int k = 0; k < gpp; ++k) s += p[k * C];
        db[co] = s;
    }
}

}  // namespace

bool wgrad_mfma_supported(const Geo &g, int cin, int cout, sp_dtype_t dt) {
    if (!(dt == SP_BF16 && cin % C == 0 && cout % C == 0 && cin <= 1024 && cout <= 1024)) return false;
    const long long base = 1LL * g.ntiles * ((g.th + PH - 1) / PH) * ((g.tw + PW - 1) / PW);
    return base * g.td < 0x7fffffffLL && 1LL * g.ph * g.pw * (cin > cout ? cin : cout) < 0x7fffffffLL;
}

size_t wgrad_mfma_ws_bytes(const Geo &g, int cin, int cout) {
    WgradArgs a;
    plan(g, cin, cout, &a);
    return static_cast<size_t>(a.ngroups) * (27 * C * C + C) * sizeof(float);
}

int launch_wgrad_mfma(const void *Px, const void *Pdz, float *dw, float *db, const Geo &g, int cin, int cout,
                      void *ws, hipStream_t s) {
    WgradArgs a;
    plan(g, cin, cout, &a);
    a.x = static_cast<const uint16_t *>(Px);
    a.dz = static_cast<const uint16_t *>(Pdz);
    a.part_w = static_cast<float *>(ws);
    a.part_b = a.part_w + static_cast<size_t>(a.ngroups) * 27 * C * C;
    a.g = g;
    const unsigned grid = static_cast<unsigned>((a.ngroups + 7) / 8 * 8);
    // more than 64 KB of dynamic LDS has to be requested explicitly
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(wgrad_mfma_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return record_hip(attr);
    hipLaunchKernelGGL(wgrad_mfma_kernel, dim3(grid), dim3(kThreads), LDS_BYTES, s, a);
    int rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    const int n = 27 * cin * cout + cout;
    hipLaunchKernelGGL(reduce_wgrad_kernel, dim3((n + 255) / 256), dim3(256), 0, s, a.part_w, a.part_b, dw, db,
                       cin, cout, a.gpp);
    return record_hip(hipGetLastError());
}

}  // namespace sp3d
