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
// 2-D variant (template parameter KD = 1; geometry flag `flat`): only the taps with kd = 1 exist (x plane D
// meets dz plane D - 1, its own slice); dw and the partials then hold 9 taps.
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
    const uint16_t *x;       // input tensor holding the first x_ca input channels (all of them if x2 is null)
    const uint16_t *x2;      // tensor holding the remaining input channels (x2_cs per voxel), or null
    const uint16_t *dz;
    float *part_w;        // [ngroups][27][32][32]
    float *part_b;        // [ngroups][32]
    Geo g;
    int x_cs, dz_cs;      // channels per voxel of x and dz
    int x_ca, x2_cs;      // two-tensor input: channels [0, x_ca) come from x, [x_ca, cin) from x2
    int nco;              // output blocks; pair p = (input chunk p / nco, output block p % nco)
    int gpp;              // workgroups per pair
    int dchunk, nd, nh, nw;
    int nitems;           // work items per pair
    int ngroups;          // real workgroups = pairs * gpp; grid is rounded up to a multiple of 8
    int fold, fold_w;     // 2-D variant, tiles narrower than half a patch: `fold` consecutive slices lie side by
                          // side in a staged plane, each in a strip of fold_w = tile width + 2 columns (1: none)
    int gather;           // 1 (direct-to-LDS kernel, 3-D): x margin voxels that have a neighbour tile are staged
                          // from that tile's interior, one tile extent further along the axis (SP_HALO_GATHER)
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Where input channels [ci0, ci0 + 32) live: tensor base, its channels per voxel and the offset inside it.
struct XSrc { const uint16_t *base; int cs, co; };
__device__ __forceinline__ XSrc x_source(const WgradArgs &a, int ci0) {
    if (a.x2 && ci0 >= a.x_ca) return XSrc{a.x2, a.x2_cs, ci0 - a.x_ca};
    return XSrc{a.x, a.x_cs, ci0};
}

// Transposing LDS read of one MFMA operand half: 16 voxels x 16 channels -> 4 voxels per lane.
__device__ __forceinline__ s16x4 tr_read(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4 *)(__attribute__((address_space(3))) char *)(p));
}

// Masked 16-byte chunk: the load goes to a safe address when the chunk is outside the plane ...
__device__ __forceinline__ uint4 ldg_clamped(bool ok, const uint16_t *p, const uint16_t *safe) {
    return *reinterpret_cast<const uint4 *>(ok ? p : safe);
}
// ... and the value is zeroed where it is consumed (after the plane's MFMAs), so that nothing waits
// for the load earlier than that.
__device__ __forceinline__ uint4 keep_if(bool ok, const uint4 &v) {
    return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
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
template <int P, int KD>   // P = D mod 4
__device__ __forceinline__ void plane_step(const char *xlane, const char *zlane, f32x4 (&acc)[27]) {
    // Software pipeline over the x rows: the fragments of row R + 1 are requested before the MFMAs
    // of row R are issued, and the scheduling barriers keep the compiler from sinking the reads
    // back down to their first use (which would expose the LDS latency once per row).
    bf16x8 zf[3][4];   // [kd][row mod 4]: rows R, R-1, R-2 in use, R+1 in flight
    bf16x8 xf[2][3];   // [row parity][kw]
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) xf[0][kw] = frag(xlane + kw * 32);
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
        if (KD == 3 || kd == 1) zf[kd][0] = frag(zlane + ((P - kd + 4) % 4) * Z_PLANE);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int R = 0; R < GR + 2; ++R) {
        if (R + 1 < GR + 2) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) xf[(R + 1) & 1][kw] = frag(xlane + ((R + 1) * XC + kw) * 32);
        }
        if (R + 1 < GR) {
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
                if (KD == 3 || kd == 1)
                    zf[kd][(R + 1) & 3] = frag(zlane + ((P - kd + 4) % 4) * Z_PLANE + (R + 1) * PW * 32);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            const int h = R - kh;
            if (h < 0 || h >= GR) continue;
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    if (KD == 1 && kd != 1) continue;
                    const int tap = (kd * 3 + kh) * 3 + kw;
                    acc[tap] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[R & 1][kw], zf[kd][h & 3], acc[tap],
                                                                       0, 0, 0);
                }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int KD>
__global__ __launch_bounds__(kThreads) void wgrad_mfma_kernel(WgradArgs a) {
    constexpr int NT = KD == 1 ? 9 : 27, T0 = KD == 1 ? 9 : 0;      // taps written, first tap of acc[] among them
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const Geo &g = a.g;
    const int per_xcd = gridDim.x >> 3;
    const int group = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (group >= a.ngroups) return;
    // Neighbouring groups - the same XCD, hence the same L2 - take the pairs of ONE share of the work items: they
    // walk the same patches at the same time, and a staged chunk of x is used by cout / 32 of them, a chunk of dz
    // by cin / 32 (a cache line of a 64-channel tensor holds both of its chunks).
    const int npairs = a.ngroups / a.gpp;
    const int pair = group % npairs, gsub = group / npairs;
    const int slot = pair * a.gpp + gsub;      // where the partial sums go: the pairs one after the other
    const XSrc xs = x_source(a, C * (pair / a.nco));
    const int x_co = xs.co, dz_co = C * (pair % a.nco);   // channel offsets of this pair
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

    const size_t xplane = static_cast<size_t>(g.ph) * g.pw * xs.cs, zplane = static_cast<size_t>(g.ph) * g.pw * a.dz_cs;
    const int xrow_elems = g.pw * xs.cs, zrow_elems = g.pw * a.dz_cs;

    // Slices side by side (2-D variant, tiles at most 15 voxels wide: one patch column block, w0 = 0).  Slices do
    // not interact, so F of them share a staged plane: strip s holds padded columns 0 .. tile width + 1 of a
    // slice, and a plane step adds F slices to the sums.  dz column Z meets x columns Z, Z + 1, Z + 2; it is
    // staged (non-zero) only where x column Z + 1 is an interior column of its strip, so all three lie in that
    // strip and no product pairs voxels of different slices.
    // Per thread: strip and padded column of its main x chunk, of its edge x chunk and of its dz chunk.
    const int F = KD == 1 ? a.fold : 1;
    int xs_m = 0, xc_m = sv, xs_e = 0, xc_e = ev, zs_m = 0, zc_m = sv + 1;
    if (F > 1) {
        xs_m = sv / a.fold_w; xc_m = sv - xs_m * a.fold_w;
        xs_e = ev / a.fold_w; xc_e = ev - xs_e * a.fold_w;
        zs_m = (sv + 1) / a.fold_w; zc_m = sv + 1 - zs_m * a.fold_w;
    }

    for (int item = gsub; item < a.nitems; item += a.gpp) {
        int t = item;
        const int pw_i = t % a.nw; t /= a.nw;
        const int ph_i = t % a.nh; t /= a.nh;
        const int pd_i = t % a.nd; t /= a.nd;
        const int tile = t;
        const int d0 = pd_i * a.dchunk, h0 = ph_i * PH, w0 = pw_i * PW;
        const int dn = min(a.dchunk, g.td - d0);
        const uint16_t *tx = xs.base + static_cast<size_t>(tile) * g.tile_vox * xs.cs + x_co;
        const uint16_t *tz = a.dz + static_cast<size_t>(tile) * g.tile_vox * a.dz_cs + dz_co;

        // source offsets inside a plane and validity (x: the interior and one voxel around it; dz: tile interior)
        const int xsrc0 = ((h0 + sr) * g.pw + w0 + xc_m) * xs.cs + c4 * 8;
        const int xsrce = ((h0 + er) * g.pw + w0 + xc_e) * xs.cs + c4 * 8;
        const int zsrc0 = ((h0 + sr + 1) * g.pw + w0 + zc_m) * a.dz_cs + c4 * 8;
        // columns: inside the tile's padded row (x) / interior (dz); folded: inside a strip that exists
        const bool xcol = F > 1 ? xs_m < F : w0 + sv < g.tw + 2;
        const bool ecol = F > 1 ? xs_e < F : w0 + ev < g.tw + 2;
        const bool zcol = F > 1 ? zs_m < F && zc_m >= 1 && zc_m <= g.tw : w0 + sv < g.tw;
        bool xok[3], zok[2];
#pragma unroll
        for (int i = 0; i < 3; ++i) xok[i] = sr + 4 * i < XR && h0 + sr + 4 * i < g.th + 2 && xcol;
        const bool eok = tid < 8 * XR && h0 + er < g.th + 2 && ecol;
#pragma unroll
        for (int i = 0; i < 2; ++i) zok[i] = h0 + sr + 4 * i < g.th && zcol;
        // folded: step S of the march stands for slices F * (S - 1) + s of the chunk on the x side (steps 0 and
        // the last meet no dz and are clamped into the chunk) and F * S + s on the dz side
        const int dsteps = F > 1 ? dn / F : dn;

        // staged chunks travel in registers from the global loads (issued before a plane's MFMAs)
        // to the LDS writes (after them)
        uint4 xs0, xs1, xs2, xs3, zs0, zs1;
#define SP3D_LDG(ok, ptr, safe) ldg_clamped(ok, ptr, safe)
#define SP3D_XSLICE(D, S_) (F > 1 ? d0 + 1 + min(max(((D) - 1) * F + (S_), 0), dn - 1) : d0 + (D))
#define SP3D_FETCH(D)                                                                  \
    do {                                                                               \
        const uint16_t *px = tx + SP3D_XSLICE(D, xs_m) * xplane;                       \
        const uint16_t *pe = tx + SP3D_XSLICE(D, xs_e) * xplane;                       \
        xs0 = SP3D_LDG(xok[0], px + xsrc0, tx);                                        \
        xs1 = SP3D_LDG(xok[1], px + xsrc0 + 4 * xrow_elems, tx);                       \
        xs2 = SP3D_LDG(xok[2], px + xsrc0 + 8 * xrow_elems, tx);                       \
        xs3 = SP3D_LDG(eok, pe + xsrce, tx);                                           \
        const bool zreal = (D) < dsteps;                                               \
        const uint16_t *pz = tz + (F > 1 ? d0 + 1 + (D) * F + zs_m : d0 + (D) + 1) * zplane; \
        zs0 = SP3D_LDG(zreal && zok[0], pz + zsrc0, tz);                               \
        zs1 = SP3D_LDG(zreal && zok[1], pz + zsrc0 + 4 * zrow_elems, tz);              \
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
        const bool zreal = (D) < dsteps;                                               \
        xs0 = keep_if(xok[0], xs0); xs1 = keep_if(xok[1], xs1);                        \
        xs2 = keep_if(xok[2], xs2); xs3 = keep_if(eok, xs3);                           \
        zs0 = keep_if(zreal && zok[0], zs0); zs1 = keep_if(zreal && zok[1], zs1);      \
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
            *reinterpret_cast<uint4 *>(zbuf + 2 * Z_PLANE + zdst0 + 4 * i * PW * 32) = make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4 *>(zbuf + 3 * Z_PLANE + zdst0 + 4 * i * PW * 32) = make_uint4(0, 0, 0, 0);
        }
        SP3D_FETCH(0);
        SP3D_COMMIT(0);
        __syncthreads();

        // x is double buffered and the dz ring has 4 slots, so plane D+1 can be written while other
        // waves still read planes D, D-1, D-2: one barrier per plane.
        const int nplanes = dsteps + 2;
        for (int D = 0; D < nplanes; D += 4) {
#pragma unroll
            for (int ph = 0; ph < 4; ++ph) {
                const int Dp = D + ph;
                if (Dp < nplanes) {
                    const bool more = Dp + 1 < nplanes;
                    if (more) SP3D_FETCH(Dp + 1);
                    const char *xl = xlane + (Dp & 1) * X_BYTES;
                    // 2-D variant: x planes 0 and dn + 1 are the D margins, which hold nothing defined (and
                    // meet no dz plane): they must not reach the matrix cores
                    if (KD == 1 && (Dp < 1 || Dp > dsteps)) {
                    } else if (ph == 0) plane_step<0, KD>(xl, zlane, acc);
                    else if (ph == 1) plane_step<1, KD>(xl, zlane, acc);
                    else if (ph == 2) plane_step<2, KD>(xl, zlane, acc);
                    else plane_step<3, KD>(xl, zlane, acc);
                    if (more) SP3D_COMMIT(Dp + 1);
                    __syncthreads();
                }
            }
        }
    }

#undef SP3D_LDG
#undef SP3D_XSLICE
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
        for (int t = T0; t < T0 + NT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[((quad * 27 + t) * 4 + i) * 64 + lane] = acc[t][i];
    }
    __syncthreads();
    if (kg == 0) {
        float *pw = a.part_w + static_cast<size_t>(slot) * NT * C * C;
#pragma unroll
        for (int t = T0; t < T0 + NT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                pw[((t - T0) * C + 16 * qi + 4 * G + i) * C + 16 * qo + p] =
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
        a.part_b[slot * C + tid] = s;
    }
}

// ---------------------------------------------------------------------------------------------
// Variant for tiles whose interior is a whole number of 8 x 32 patches: every staged chunk is real
// data, so the planes go from global memory straight into LDS (global_load_lds: lane l's 16 bytes
// land at LDS base + 16*l) two planes ahead of their use, and no registers, LDS writes or VALU work
// are spent on staging.  What the staging registers did for free moves elsewhere:
//  - dz planes outside the D chunk (D - kd < 0 or >= dn) are not zero-filled in LDS; the fragments
//    read for such a plane are and-ed with a wave-uniform zero mask instead, so stale LDS contents
//    (any bit pattern) never reach the matrix cores;
//  - the bias gradient is one more MFMA per dz row with an all-ones A operand (every row of the
//    result is the column sum), issued by one wave per SIMD.
constexpr int NXB = 3, NZB = 5;               // ring slots: x planes D..D+2, dz planes D-2..D+2
constexpr int XG = (XVOX + 31) / 32;          // 11 groups of 32 voxels per x plane; the last one is padded
constexpr int XD_HALF = XG * 32 * 32 + 64;    // 11328: room for the padding voxels of the last group
constexpr int XD_BYTES = 2 * XD_HALF;
constexpr int DMA_STAGE_BYTES = NXB * XD_BYTES + NZB * Z_PLANE;       // 150528
constexpr int DMA_LDS_BYTES = DMA_STAGE_BYTES > RED_BYTES ? DMA_STAGE_BYTES : RED_BYTES;
static_assert(DMA_LDS_BYTES <= 160 * 1024, "LDS of one CU");
// Wave loads per plane pair: 2 halves x 11 groups for x, 2 halves x 8 groups for dz.  Each of the 8
// waves issues 3 x loads (24 slots for 22 loads: the last two waves repeat one of theirs) and 2 dz loads.
constexpr int DMA_X = 3, DMA_Z = 2, DMA_PER_WAVE = DMA_X + DMA_Z;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at dst + 16*l (dst is
// wave-uniform and travels in M0).  Written as assembly because the compiler, when it knows of such a
// load, waits for ALL outstanding ones before every transposing LDS read, which would undo the
// two-plane prefetch; the kernel waits for exactly the loads it needs with explicit s_waitcnt vmcnt.
__device__ __forceinline__ void dma16(const uint16_t *src, char *dst) {
    const uint32_t l = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) char *)dst));
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(src), "s"(l)
                 : "memory");
}

__device__ __forceinline__ bf16x8 frag_masked(const char *p, uint32_t m) {
    union { struct { s16x4 lo, hi; } s; u32x4 w; bf16x8 v; } u;
    u.s.lo = tr_read(p);
    u.s.hi = tr_read(p + 16 * 32);
    u.w &= m;
    return u.v;
}

// Same march as plane_step, with run-time ring slots: z[kd] points at dz plane D - kd, m[kd] is
// all ones if that plane exists and zero otherwise.
template <int KD>
__device__ __forceinline__ void plane_step_dma(const char *xl, const char *z0, const char *z1, const char *z2,
                                               uint32_t m0, uint32_t m1, uint32_t m2, bool bias_wave,
                                               f32x4 (&acc)[27], f32x4 &accb) {
    const char *z[3] = {z0, z1, z2};
    const uint32_t m[3] = {m0, m1, m2};
    union { uint32_t w[4]; bf16x8 v; } ones;
#pragma unroll
    for (int i = 0; i < 4; ++i) ones.w[i] = 0x3f803f80u;     // bf16 1.0 pairs
    bf16x8 zf[3][4];
    bf16x8 xf[2][3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) xf[0][kw] = frag(xl + kw * 32);
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
        if (KD == 3 || kd == 1) zf[kd][0] = frag_masked(z[kd], m[kd]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int R = 0; R < GR + 2; ++R) {
        if (R + 1 < GR + 2) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) xf[(R + 1) & 1][kw] = frag(xl + ((R + 1) * XC + kw) * 32);
        }
        if (R + 1 < GR) {
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
                if (KD == 3 || kd == 1) zf[kd][(R + 1) & 3] = frag_masked(z[kd] + (R + 1) * PW * 32, m[kd]);
        }
        __builtin_amdgcn_sched_barrier(0);
        // every dz plane passes once through each kd position (masked when it does not exist); the 2-D
        // variant only reads position 1
        if (bias_wave && R < GR)      // wave-uniform
            accb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones.v, zf[KD == 1 ? 1 : 0][R & 3], accb, 0, 0, 0);
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            const int h = R - kh;
            if (h < 0 || h >= GR) continue;
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    if (KD == 1 && kd != 1) continue;
                    const int tap = (kd * 3 + kh) * 3 + kw;
                    acc[tap] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[R & 1][kw], zf[kd][h & 3], acc[tap],
                                                                       0, 0, 0);
                }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The same step (x, z[kd]: this lane's read bases in x plane D and in dz planes D - kd; m[kd] as above) cut in two so that the
// workgroup's barrier can stand inside it: rows R0 .. R1 - 1 of the x plane; the fragments of row R0 are in
// xf / zf already (read by the previous call), and the call reads those of row R1 - or, for the last row, those of
// row 0 of the NEXT plane (nx) - before its last row's MFMAs.  Rows 0 and GR + 1 carry 9 MFMAs against 12 fragment
// reads, so at a plane boundary that begins with a barrier and reads from scratch the matrix cores wait out the
// LDS latency with nothing to do; with the barrier behind row GR - 1 and the next plane's first fragments on
// their way during row GR + 1 the rows follow each other without a gap.
struct DmaPlane { const char *x; const char *z[3]; uint32_t m[3]; };
template <int KD>
__device__ __forceinline__ void dma_row0(const DmaPlane &pl, bf16x8 (&xf)[2][3], bf16x8 (&zf)[3][4]) {
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) xf[0][kw] = frag(pl.x + kw * 32);
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
        if (KD == 3 || kd == 1) zf[kd][0] = frag_masked(pl.z[kd], pl.m[kd]);
}
template <int KD, int R0, int R1>
__device__ __forceinline__ void plane_rows_dma(const DmaPlane &pl, const DmaPlane &nx, bool bias_wave,
                                               bf16x8 (&xf)[2][3], bf16x8 (&zf)[3][4], f32x4 (&acc)[27],
                                               f32x4 &accb) {
    union { uint32_t w[4]; bf16x8 v; } ones;
#pragma unroll
    for (int i = 0; i < 4; ++i) ones.w[i] = 0x3f803f80u;     // bf16 1.0 pairs
    static_assert(((GR + 2) & 1) == 0 && GR == 4, "row GR + 1 reads the next plane's row 0 into buffer 0 / ring slot 0");
#pragma unroll
    for (int R = R0; R < R1; ++R) {
        if (R + 1 < GR + 2) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) xf[(R + 1) & 1][kw] = frag(pl.x + ((R + 1) * XC + kw) * 32);
            if (R + 1 < GR) {
#pragma unroll
                for (int kd = 0; kd < 3; ++kd)
                    if (KD == 3 || kd == 1)
                        zf[kd][(R + 1) & 3] = frag_masked(pl.z[kd] + (R + 1) * PW * 32, pl.m[kd]);
            }
        } else {
            dma_row0<KD>(nx, xf, zf);      // row GR + 1 uses xf[1] and ring slot GR - 1 only
        }
        __builtin_amdgcn_sched_barrier(0);
        // every dz plane passes once through each kd position (masked when it does not exist); the 2-D
        // variant only reads position 1
        if (bias_wave && R < GR)      // wave-uniform
            accb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones.v, zf[KD == 1 ? 1 : 0][R & 3], accb, 0, 0, 0);
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            const int h = R - kh;
            if (h < 0 || h >= GR) continue;
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    if (KD == 1 && kd != 1) continue;
                    const int tap = (kd * 3 + kh) * 3 + kw;
                    acc[tap] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[R & 1][kw], zf[kd][h & 3], acc[tap],
                                                                       0, 0, 0);
                }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// MID: the march with the barrier inside the step (see plane_rows_dma and the loop below); otherwise the barrier
// ends the step.
template <int KD, bool MID>
__global__ __launch_bounds__(kThreads) void wgrad_mfma_dma_kernel(WgradArgs a) {
    constexpr int NT = KD == 1 ? 9 : 27, T0 = KD == 1 ? 9 : 0;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const Geo &g = a.g;
    const int per_xcd = gridDim.x >> 3;
    const int group = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (group >= a.ngroups) return;
    // Neighbouring groups - the same XCD, hence the same L2 - take the pairs of ONE share of the work items: they
    // walk the same patches at the same time, and a staged chunk of x is used by cout / 32 of them, a chunk of dz
    // by cin / 32 (a cache line of a 64-channel tensor holds both of its chunks).
    const int npairs = a.ngroups / a.gpp;
    const int pair = group % npairs, gsub = group / npairs;
    const int slot = pair * a.gpp + gsub;      // where the partial sums go: the pairs one after the other
    const XSrc xs = x_source(a, C * (pair / a.nco));
    const int x_co = xs.co, dz_co = C * (pair % a.nco);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: scalar control flow below
    // Waves w and w + 4 share a SIMD: give them different ci halves, so that each SIMD hosts exactly one
    // of the four waves (ci half 0) that also accumulate the bias gradient.
    const int kg = wave >> 2;
    const int qo = wave & 1, qi = ((wave >> 1) & 1) ^ kg;
    const bool bias_wave = qi == 0;
    char *xbuf = lds;
    char *zbuf = lds + NXB * XD_BYTES;
    const int G = lane >> 4, p = lane & 15;
    const int lane_off = (4 * G + (p >> 2)) * 32 + (p & 3) * 8;
    const char *xlane = xbuf + qi * XD_HALF + lane_off + kg * GR * XC * 32;
    const char *zlane = zbuf + qo * Z_HALF + lane_off + kg * GR * PW * 32;

    // Staging loads of this wave: x loads u = 2*wave, 2*wave + 1 and 16 + wave (waves 6, 7 repeat their
    // second one), dz loads 2*wave, 2*wave + 1.  Load u covers half u / groups, voxel group u % groups;
    // lane l fetches chunk l & 1 of voxel 32*group + l/2.  Voxels past the end of the x plane (last
    // group) re-fetch its last voxel into the padding.
    int gx[DMA_X], gz[DMA_Z];        // source offsets (elements) inside the item's plane
    int lx[DMA_X], lz[DMA_Z];        // LDS byte offsets inside ring slot 0
#pragma unroll
    for (int j = 0; j < DMA_X; ++j) {
        const int u = j < 2 ? 2 * wave + j : (wave < 6 ? 16 + wave : 2 * wave + 1);
        const int half = u / XG, vg = u % XG;
        const int v = min(vg * 32 + (lane >> 1), XVOX - 1);
        gx[j] = ((v / XC) * g.pw + v % XC) * xs.cs + half * 16 + (lane & 1) * 8;
        lx[j] = half * XD_HALF + vg * 1024;
    }
#pragma unroll
    for (int j = 0; j < DMA_Z; ++j) {
        const int u = 2 * wave + j;
        const int half = u / (ZVOX / 32), vg = u % (ZVOX / 32);
        const int v = vg * 32 + (lane >> 1);
        gz[j] = ((v / PW + 1) * g.pw + v % PW + 1) * a.dz_cs + half * 16 + (lane & 1) * 8;
        lz[j] = NXB * XD_BYTES + half * Z_HALF + vg * 1024;
    }

    f32x4 acc[27];
#pragma unroll
    for (int t = 0; t < 27; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 accb = f32x4{0.f, 0.f, 0.f, 0.f};

    const size_t xplane = static_cast<size_t>(g.ph) * g.pw * xs.cs, zplane = static_cast<size_t>(g.ph) * g.pw * a.dz_cs;

    int sx = 0, sz = 0;       // ring slots of the plane in use; the rings turn on from item to item
    for (int item = gsub; item < a.nitems; item += a.gpp) {
        int t = item;
        const int pw_i = t % a.nw; t /= a.nw;
        const int ph_i = t % a.nh; t /= a.nh;
        const int pd_i = t % a.nd; t /= a.nd;
        const int tile = t;
        const int d0 = pd_i * a.dchunk, h0 = ph_i * PH, w0 = pw_i * PW;
        const int dn = min(a.dchunk, g.td - d0);
        // padded plane d0 of the tile, at the patch's first voxel and the pair's channels
        const uint16_t *tx = xs.base + (static_cast<size_t>(tile) * g.tile_vox + static_cast<size_t>(d0) * g.ph * g.pw +
                                        h0 * g.pw + w0) * xs.cs + x_co;
        const uint16_t *tz = a.dz + (static_cast<size_t>(tile) * g.tile_vox + static_cast<size_t>(d0 + 1) * g.ph * g.pw +
                                     h0 * g.pw + w0) * a.dz_cs + dz_co;

        // Gathered halos: a margin voxel of x that the exchange would have filled is, in the neighbour tile, the
        // interior voxel one tile extent further along the axis.  Along H and W that is a per-lane constant for
        // this item's patch (gxa), along D a uniform one for the item's first / last x plane (dlo, dhi).  Margins
        // at the volume border are read from the tensor itself (zero padding).
        int gxa[DMA_X];
        ptrdiff_t dlo = 0, dhi = 0;
#pragma unroll
        for (int j = 0; j < DMA_X; ++j) gxa[j] = gx[j];
        if (a.gather) {
            const int tc = tile % g.gw, t1 = tile / g.gw;
            const int tb = t1 % g.gh, ta = (t1 / g.gh) % g.gd;
            const ptrdiff_t tv = static_cast<ptrdiff_t>(g.tile_vox);
            const ptrdiff_t sw = (tv - g.tw) * xs.cs;
            const ptrdiff_t sh = (tv * g.gw - static_cast<ptrdiff_t>(g.th) * g.pw) * xs.cs;
            const ptrdiff_t sd = (tv * g.gw * g.gh - static_cast<ptrdiff_t>(g.td) * g.ph * g.pw) * xs.cs;
#pragma unroll
            for (int j = 0; j < DMA_X; ++j) {
                const int u = j < 2 ? 2 * wave + j : (wave < 6 ? 16 + wave : 2 * wave + 1);
                const int v = min((u % XG) * 32 + (lane >> 1), XVOX - 1);
                const int row = h0 + v / XC, col = w0 + v % XC;
                gxa[j] += (row == 0 && tb > 0 ? static_cast<int>(-sh) : 0) +
                          (row == g.th + 1 && tb < g.gh - 1 ? static_cast<int>(sh) : 0) +
                          (col == 0 && tc > 0 ? static_cast<int>(-sw) : 0) +
                          (col == g.tw + 1 && tc < g.gw - 1 ? static_cast<int>(sw) : 0);
            }
            if (d0 == 0 && ta > 0) dlo = -sd;
            if (d0 + dn == g.td && ta < g.gd - 1) dhi = sd;
        }

        // Stage planes D of x and dz into ring slots sx, sz.  Planes past the last one are clamped to it:
        // their slots are either never read or masked, and every call issues exactly DMA_PER_WAVE loads.
#define SP3D_STAGE(D, sx, sz)                                                                      \
    do {                                                                                           \
        const int dx_ = min((D), dn + 1);                                                          \
        const uint16_t *px = tx + dx_ * xplane + (dx_ == 0 ? dlo : 0) + (dx_ == dn + 1 ? dhi : 0); \
        const uint16_t *pz = tz + min((D), dn - 1) * zplane;                                       \
        _Pragma("unroll") for (int j = 0; j < DMA_X; ++j) dma16(px + gxa[j], lds + lx[j] + (sx) * XD_BYTES); \
        _Pragma("unroll") for (int j = 0; j < DMA_Z; ++j) dma16(pz + gz[j], lds + lz[j] + (sz) * Z_PLANE);  \
    } while (0)

        if (MID) {
            // The item's march.  Step D: rows 0 .. GR - 1 of x plane D; wait + barrier; stage planes D + 2; rows GR, GR + 1,
            // during which row 0 of plane D + 1 is read.  At the barrier every wave has finished step D - 1, whose
            // last rows read x plane D - 1 and dz plane D - 3: the slots that planes D + 2 go to, which is why the
            // staging stands behind it; and plane D + 1 (staged behind the previous step's barrier, a whole step ago)
            // has landed when this wave's own loads are done (vmcnt(0): nothing younger is in flight) and every other
            // wave says the same.  The last two steps of an item stage its last plane again (clamped) into the two slots
            // behind that plane's in both rings; the next item's first two planes go to the same slots, with no barrier
            // in between: waves still in the last rows of this item read other slots, and a wave's loads land in order.
            SP3D_STAGE(0, sx, sz);
            SP3D_STAGE(1, (sx + 1 == NXB ? 0 : sx + 1), (sz + 1 == NZB ? 0 : sz + 1));
            asm volatile("s_waitcnt vmcnt(5)" ::: "memory");      // plane 0
            __builtin_amdgcn_s_barrier();

            const int nplanes = dn + 2;
            bf16x8 xf[2][3], zf[3][4];
            auto plane_at = [&](int D, int sxD, int szD) {
                const int sz1 = szD == 0 ? NZB - 1 : szD - 1;
                const int sz2m = sz1 == 0 ? NZB - 1 : sz1 - 1;
                DmaPlane pl;
                pl.x = xlane + sxD * XD_BYTES;
                pl.z[0] = zlane + szD * Z_PLANE; pl.z[1] = zlane + sz1 * Z_PLANE; pl.z[2] = zlane + sz2m * Z_PLANE;
                pl.m[0] = D < dn ? 0xffffffffu : 0u;
                pl.m[1] = (D >= 1 && D - 1 < dn) ? 0xffffffffu : 0u;
                pl.m[2] = D >= 2 ? 0xffffffffu : 0u;
                return pl;
            };
            DmaPlane cur = plane_at(0, sx, sz);
            dma_row0<KD>(cur, xf, zf);
            for (int D = 0; D < nplanes; ++D) {
                const int sxn = sx + 1 == NXB ? 0 : sx + 1, szn = sz + 1 == NZB ? 0 : sz + 1;
                const DmaPlane nxt = plane_at(D + 1, sxn, szn);
                // (2-D variant: x planes 0 and dn + 1 are the undefined D margins and meet no dz plane; their
                // rows are skipped but the fragments of the next plane's first row are still read)
                const bool live = KD == 3 || (D >= 1 && D <= dn);
                if (live) plane_rows_dma<KD, 0, GR>(cur, nxt, bias_wave, xf, zf, acc, accb);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                {
                    const int sx2 = sx + 2 >= NXB ? sx + 2 - NXB : sx + 2;
                    const int sz2 = sz + 2 >= NZB ? sz + 2 - NZB : sz + 2;
                    SP3D_STAGE(D + 2, sx2, sz2);
                }
                if (live) plane_rows_dma<KD, GR, GR + 2>(cur, nxt, bias_wave, xf, zf, acc, accb);
                else dma_row0<KD>(nxt, xf, zf);
                cur = nxt;
                sx = sxn;
                sz = szn;
            }
        } else {
            // every wave has left the previous item's last plane (the barrier that ended it)
            SP3D_STAGE(0, 0, 0);
            SP3D_STAGE(1, 1, 1);
            asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
            __builtin_amdgcn_s_barrier();

            const int nplanes = dn + 2;
            sx = 0; sz = 0;                   // ring slots of planes D
            for (int D = 0; D < nplanes; ++D) {
                {
                    const int sx2 = sx + 2 >= NXB ? sx + 2 - NXB : sx + 2;
                    const int sz2 = sz + 2 >= NZB ? sz + 2 - NZB : sz + 2;
                    SP3D_STAGE(D + 2, sx2, sz2);
                }
                const int sz1 = sz == 0 ? NZB - 1 : sz - 1;
                const int sz2m = sz1 == 0 ? NZB - 1 : sz1 - 1;
                const uint32_t m0 = D < dn ? 0xffffffffu : 0u;
                const uint32_t m1 = (D >= 1 && D - 1 < dn) ? 0xffffffffu : 0u;
                const uint32_t m2 = D >= 2 ? 0xffffffffu : 0u;
                // (2-D variant: x planes 0 and dn + 1 are the undefined D margins and meet no dz plane)
                if (KD == 3 || (D >= 1 && D <= dn))
                    plane_step_dma<KD>(xlane + sx * XD_BYTES, zlane + sz * Z_PLANE, zlane + sz1 * Z_PLANE,
                               zlane + sz2m * Z_PLANE, m0, m1, m2, bias_wave, acc, accb);
                // plane D + 1 (staged one step ago) has landed once at most this step's loads are in flight
                asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                sx = sx + 1 == NXB ? 0 : sx + 1;
                sz = sz + 1 == NZB ? 0 : sz + 1;
            }
        }
    }
#undef SP3D_STAGE

    // The clamped loads of the last item may still be writing LDS: drain them before the staging area is
    // reused for the reductions.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    float *red = reinterpret_cast<float *>(lds);
    const int quad = qi * 2 + qo;
    if (kg == 1) {
#pragma unroll
        for (int t = T0; t < T0 + NT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[((quad * 27 + t) * 4 + i) * 64 + lane] = acc[t][i];
    }
    __syncthreads();
    if (kg == 0) {
        float *pw = a.part_w + static_cast<size_t>(slot) * NT * C * C;
#pragma unroll
        for (int t = T0; t < T0 + NT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                pw[((t - T0) * C + 16 * qi + 4 * G + i) * C + 16 * qo + p] =
                    acc[t][i] + red[((quad * 27 + t) * 4 + i) * 64 + lane];
    }
    // bias partial: row 0 of the ones-product (lanes 0..15, register 0) holds the column sums of the
    // wave's co half and row group
    __syncthreads();
    if (bias_wave && lane < 16) red[(kg * 2 + qo) * 16 + lane] = accb[0];
    __syncthreads();
    if (tid < C) a.part_b[slot * C + tid] = red[tid] + red[C + tid];
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
    // 2-D variant, tiles narrower than half a patch: up to 4 slices side by side in a staged plane; the tile's
    // slice count and the D chunk must be multiples of that number (only the register-staged kernel folds: such
    // tiles are never whole patches)
    a->fold = 1;
    a->fold_w = g.tw + 2;
    if (g.flat && 2 * (g.tw + 2) <= XC) {
        int f = XC / (g.tw + 2);
        if (f > 4) f = 4;
        while (f > 1 && g.td % f) --f;
        a->fold = f;
        dchunk = (dchunk + f - 1) / f * f;
    }
    a->dchunk = dchunk;
    a->nd = (g.td + dchunk - 1) / dchunk;
    const long long items = base * a->nd;
    a->nitems = static_cast<int>(items);
    a->gpp = static_cast<int>(items < gpp ? items : gpp);
    a->ngroups = a->gpp * npairs;
}

// dw[tap][ci][co] = sum over the workgroups of pair (ci/32, co/32) of their partial [tap][ci%32][co%32];
// db[co] likewise from the pairs of input chunk 0.  Eight neighbouring lanes share one output: lane s adds
// the contiguous run of workgroups [s*gpp/8, (s+1)*gpp/8) in order, and the eight run sums are combined by
// a fixed three-level tree, so the grouping depends only on gpp and the result is reproducible.  (One
// serial chain of gpp dependent loads per output was latency-bound: 72 us for 28 MB of partials.)
// With fewer than eight workgroups per pair (wide layers: a pair per workgroup) one lane adds them all:
// seven idle lanes per output made the plain re-layout of a 1024 x 1024 layer's 38 MB cost 0.24 ms.
template <int RSPLIT>
__global__ __launch_bounds__(256) void reduce_wgrad_kernel(const float *__restrict__ part_w,
                                                           const float *__restrict__ part_b,
                                                           float *__restrict__ dw, float *__restrict__ db,
                                                           int cin, int cout, int gpp, int ntaps) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int e = t / RSPLIT, sub = t % RSPLIT;
    const int nw_ = ntaps * cin * cout;
    const size_t gstride = static_cast<size_t>(ntaps) * C * C;      // partial of one workgroup
    const int k0 = static_cast<int>(1LL * sub * gpp / RSPLIT), k1 = static_cast<int>(1LL * (sub + 1) * gpp / RSPLIT);
    float s = 0.f;
    if (e < nw_) {
        const int co = e % cout, ci = (e / cout) % cin, tap = e / (cout * cin);
        const int pair = (ci / C) * (cout / C) + co / C;
        const float *p = part_w + (static_cast<size_t>(pair) * gpp * ntaps + tap) * C * C + (ci % C) * C + co % C;
        int k = k0;
        for (; k + 4 <= k1; k += 4) {          // loads issued together, additions kept in order
            const float p0 = p[k * gstride], p1 = p[(k + 1) * gstride];
            const float p2 = p[(k + 2) * gstride], p3 = p[(k + 3) * gstride];
            s = (((s + p0) + p1) + p2) + p3;
        }
        for (; k < k1; ++k) s += p[k * gstride];
    } else if (e < nw_ + cout) {
        const int co = e - nw_;
        const float *p = part_b + static_cast<size_t>(co / C) * gpp * C + co % C;     // pairs (0, co/32)
        for (int k = k0; k < k1; ++k) s += p[k * C];
    }
    // lanes 8j .. 8j+7 hold the run sums of one output (every lane of the wave takes part in the shuffles)
    if (RSPLIT == 8) {
        s += __shfl_xor(s, 1);
        s += __shfl_xor(s, 2);
        s += __shfl_xor(s, 4);
    }
    if (sub == 0) {
        if (e < nw_) dw[e] = s;
        else if (db && e < nw_ + cout) db[e - nw_] = s;
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
    return static_cast<size_t>(a.ngroups) * (taps_of(g) * C * C + C) * sizeof(float);
}

bool wgrad_mfma_gather_supported(const Geo &g, int cin, int cout, sp_dtype_t dt) {
    // the direct-to-LDS kernel (whole patches), one-voxel margins, 3-D; per-lane offsets to the H / W neighbours
    // (and their sum at an edge) must fit the 32-bit staging offsets
    return wgrad_mfma_supported(g, cin, cout, dt) && g.halo == 1 && !g.flat && g.th % PH == 0 && g.tw % PW == 0 &&
           static_cast<long long>(g.tile_vox) * (g.gw + 1) * cin < 0x7fffffffLL;
}

int launch_wgrad_mfma(const void *Px, const void *Pdz, float *dw, float *db, const Geo &g, int cin, int cout,
                      void *ws, hipStream_t s, const void *Px2, int ca, bool gather) {
    if (gather && !wgrad_mfma_gather_supported(g, cin, cout, SP_BF16)) return SP_EUNSUPPORTED;
    WgradArgs a;
    plan(g, cin, cout, &a);
    a.gather = gather ? 1 : 0;
    a.x = static_cast<const uint16_t *>(Px);
    a.x2 = static_cast<const uint16_t *>(Px2);
    if (Px2) { a.x_cs = ca; a.x_ca = ca; a.x2_cs = cin - ca; }
    else { a.x_ca = cin; a.x2_cs = 0; }
    a.dz = static_cast<const uint16_t *>(Pdz);
    a.part_w = static_cast<float *>(ws);
    const int ntaps = taps_of(g);
    a.part_b = a.part_w + static_cast<size_t>(a.ngroups) * ntaps * C * C;
    a.g = g;
    const unsigned grid = static_cast<unsigned>((a.ngroups + 7) / 8 * 8);
    // more than 64 KB of dynamic LDS has to be requested explicitly
    using Kern = void (*)(WgradArgs);
    static const Kern plain[2] = {wgrad_mfma_kernel<3>, wgrad_mfma_kernel<1>};          // [2-D variant]
    static const Kern dma[2][2] = {{wgrad_mfma_dma_kernel<3, false>, wgrad_mfma_dma_kernel<1, false>},
                                   {wgrad_mfma_dma_kernel<3, true>, wgrad_mfma_dma_kernel<1, true>}};      // [MID][2-D variant]
    static const hipError_t attr = [] {
        for (int i = 0; i < 2; ++i) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(plain[i]),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
            if (e != hipSuccess) return e;
            for (int m = 0; m < 2; ++m) {
                e = hipFuncSetAttribute(reinterpret_cast<const void *>(dma[m][i]),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, DMA_LDS_BYTES);
                if (e != hipSuccess) return e;
            }
        }
        return hipSuccess;
    }();
    if (attr != hipSuccess) return record_hip(attr);
    // whole patches only: the direct-to-LDS loads cannot zero-fill a ragged edge
    // The march with the barrier inside the step has no idle matrix cores at a plane boundary but stages one step
    // ahead where the other stages two (the rings have no slot for more).  Measured: it wins where a launch has few
    // channel pairs (32 -> 32 at 512^3: 6.00 -> 5.79 ms; 64 -> 64: -2 %) and loses from 16 pairs on (128 channels
    // + 1 %, 256 + 5 %, 512 + 6 %), where many workgroups stream different planes at once and a plane takes longer
    // to arrive than a step lasts.
    const int mid = (cin / C) * (cout / C) <= 4 ? 1 : 0;
    if (g.th % PH == 0 && g.tw % PW == 0)
        hipLaunchKernelGGL(dma[mid][g.flat], dim3(grid), dim3(kThreads), DMA_LDS_BYTES, s, a);
    else
        hipLaunchKernelGGL(plain[g.flat], dim3(grid), dim3(kThreads), LDS_BYTES, s, a);
    int rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    const int rsplit = a.gpp >= 8 ? 8 : 1;
    const long long n = (1LL * ntaps * cin * cout + cout) * rsplit;
    const dim3 rgrid(static_cast<unsigned>((n + 255) / 256));
    if (rsplit == 8)
        hipLaunchKernelGGL(reduce_wgrad_kernel<8>, rgrid, dim3(256), 0, s, a.part_w, a.part_b, dw, db, cin, cout,
                           a.gpp, ntaps);
    else
        hipLaunchKernelGGL(reduce_wgrad_kernel<1>, rgrid, dim3(256), 0, s, a.part_w, a.part_b, dw, db, cin, cout,
                           a.gpp, ntaps);
    return record_hip(hipGetLastError());
}

}  // namespace sp3d
