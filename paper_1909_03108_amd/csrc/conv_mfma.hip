// bf16 implicit-GEMM 3x3x3 convolution on padded tiles for Cin = Cout = 32, on the gfx950 matrix
// cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).  Serves conv3d_fwd and, with mirrored taps
// and swapped channel roles, conv3d_dgrad.
//
// Work decomposition.  A workgroup (4 waves, one per SIMD) owns an output patch of 8 rows (H) x 32
// columns (W) of one tile and marches along D.  Each input plane (10 x 34 voxels x 32 channels) is
// staged once in LDS by direct global->LDS loads, three planes ahead of the plane being consumed
// (ring of four).  A wave owns 2 of the 8 rows and keeps the accumulators of consecutive output
// planes in registers: input plane D feeds output planes D, D-1, D-2 through taps kd = 0, 1, 2, so an
// input fragment read from LDS once is used by up to 3 (kd) x 2 (kh) MFMAs.  A fourth accumulator
// slot holds the plane finished in the previous step, whose conversion and stores are spread over
// the MFMA stream of the current step.  All 27 x 2 weight fragments (32 x 16 each) live in
// registers for the whole march.
//
// MFMA operand roles: A = weights [M = Cout][K = 16 input channels], B = voxels [K][N = 32 voxels
// along W], D[M = Cout][N = voxel].  Lane l of B supplies voxel l%32, channels 8*(l/32)..+7 of the
// 16-channel half; lane l of D holds voxel l%32, channels 8*(i/4) + 4*(l/32) + i%4 for i = 0..15.
#include "common.h"

#include <type_traits>

namespace sp3d {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int C = 32;                       // channels in and out
constexpr int kWaves = 4, kThreads = 256;
constexpr int RH = 2;                       // output rows per wave
constexpr int PH = RH * kWaves;             // patch rows
constexpr int PW = 32;                      // patch columns = MFMA N
constexpr int LROWS = PH + 2, LCOLS = PW + 2;
constexpr int PLANE_VOX = LROWS * LCOLS;    // 340
constexpr int LOADS = (PLANE_VOX + 63) / 64;   // wave-wide staging loads per chunk plane: 6
constexpr int NBUF = 4;                     // LDS ring of staged planes
constexpr int DIST = 3;                     // planes fetched ahead of the one being consumed
constexpr int NFRAG = 27 * 2;               // weight fragments per lane (16 bytes each)
constexpr int NG = 6;                       // (kw, K-half) groups per plane
static_assert(LOADS == NG, "one staging load is issued per MFMA group");

// LDS layout of a staged plane: four chunk planes (16-byte chunk c of every voxel record), each an
// array of 16-byte entries indexed by the patch-local voxel.  A fragment read (32 consecutive voxels,
// same chunk) is then 512 contiguous bytes per half wave, and every read address is one per-lane base
// plus a compile-time offset.
constexpr int CH_STRIDE = (PLANE_VOX + 2) * 16;     // 5472 bytes
constexpr int PLANE_BYTES = 4 * CH_STRIDE;          // 21888 bytes
constexpr int LDS_BYTES = NBUF * PLANE_BYTES;       // 87552 bytes
__device__ __forceinline__ int lds_off(int v, int c) { return c * CH_STRIDE + v * 16; }

struct ConvArgs {
    const uint16_t *in;
    const uint4 *wpack;     // [27][2][64] fragments of 16 bytes
    const float *bias;
    uint16_t *out;
    Geo g;
    int dchunk;             // output planes per workgroup
    int nd, nh, nw;         // patches per tile along D, H, W
    int nblocks;            // real workgroups (grid is rounded up to a multiple of 8)
    int relu;
};

// Pre-swizzle the weights into MFMA A-fragment order: wpack[tap][half][lane] = the 8 input
// channels k = 16*half + 8*(lane/32) + j of output channel m = lane%32.
// Forward reads w[tap][k][m]; data-grad reads w[26-tap][m][k] (taps mirrored, roles swapped).
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t *__restrict__ w,
                                                           uint16_t *__restrict__ wpack, int dgrad) {
    const int i = blockIdx.x * 256 + threadIdx.x;     // over 27*2*64*8 elements
    if (i >= NFRAG * 64 * 8) return;
    const int j = i & 7, lane = (i >> 3) & 63, half = (i >> 9) & 1, tap = i >> 10;
    const int m = lane & 31, k = 16 * half + 8 * (lane >> 5) + j;
    wpack[i] = dgrad ? w[((26 - tap) * C + m) * C + k] : w[(tap * C + k) * C + m];
}

// two floats -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack2(float a, float b) {
    union { bf16x2 v; uint32_t u; } r;
    r.v = __builtin_convertvector(f32x2{a, b}, bf16x2);
    return r.u;
}

// Per-wave state of the march that the side work of a step needs.
template <bool HAS_BIAS>
struct Ctx {
    const uint16_t *tin0;       // first padded input plane of this workgroup's D chunk
    size_t plane_elems;         // elements per padded plane of the tile
    int nplanes;                // input planes of the chunk (output planes + 2)
    int goff[LOADS];            // per-lane source offsets of the staging loads (elements)
    char *lds_stage;            // LDS chunk plane this wave fills (ring slot 0)
    uint16_t *obase;            // output address of (plane 0, first row of the wave, this lane)
    size_t orow;                // elements per padded row
    bool okrow[RH];             // row/column of this lane lies inside the tile interior
    float bv[HAS_BIAS ? 16 : 1];
};

// Staging load j of padded plane `dplane` of the chunk -> ring slot dplane % NBUF.  global_load_lds:
// lane l supplies its own global address and the 16 bytes land at LDS base + 16*l.  Planes past the last
// one needed are clamped (their ring slot is never read), so every step issues exactly LOADS loads.
template <bool HAS_BIAS>
__device__ __forceinline__ void stage(const Ctx<HAS_BIAS> &c, int dplane, int j, int lane) {
    const uint16_t *p = c.tin0 + min(dplane, c.nplanes - 1) * c.plane_elems;
    char *dst = c.lds_stage + (dplane % NBUF) * PLANE_BYTES + j * 1024;
    if (64 * j + lane < PLANE_VOX)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p + c.goff[j]),
                                         (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
}

// Convert and store 4 channels (8 bytes) of row h of a finished plane: channels 8q + 4*(lane/32) .. +3.
template <bool RELU, bool FULL, bool HAS_BIAS>
__device__ __forceinline__ void store_unit(const Ctx<HAS_BIAS> &c, int d, const f32x16 (&s)[RH], int h, int q) {
    float v0 = s[h][4 * q], v1 = s[h][4 * q + 1], v2 = s[h][4 * q + 2], v3 = s[h][4 * q + 3];
    if (RELU) {
        v0 = v0 < 0.f ? 0.f : v0; v1 = v1 < 0.f ? 0.f : v1;
        v2 = v2 < 0.f ? 0.f : v2; v3 = v3 < 0.f ? 0.f : v3;
    }
    const uint2 pk = make_uint2(pack2(v0, v1), pack2(v2, v3));
    uint2 *o = reinterpret_cast<uint2 *>(c.obase + d * c.plane_elems + h * c.orow + 8 * q);
    if (FULL || c.okrow[h]) *o = pk;
}

// All MFMAs of one staged input plane Dp, with the step's side work spread over the six MFMA groups:
// the staging loads of plane Dp+DIST and (EPI) the conversion and stores of output plane Dp-3, which
// received its last contribution in step Dp-1, after which its accumulator slot returns to the bias.
// `lbase` = this lane's read base inside the plane: voxel (first row of the wave, column lane%32),
// chunk lane/32.  Fragments are fetched one (kw, K-half) group of RH+2 rows ahead of the MFMAs that
// consume them.  P = Dp mod 4: output plane Dp-kd lives in slot (P-kd) mod 4, plane Dp-3 in slot (P+1) mod 4.
// FULL: the patch lies completely inside the tile interior, so stores need no mask (no branches in
// the step, which lets the scheduler weave the side work between the MFMAs).
template <int P, bool EPI, bool RELU, bool FULL, bool HAS_BIAS>
__device__ __forceinline__ void plane_step(const Ctx<HAS_BIAS> &c, int Dp, int lane, const char *lbase,
                                           const bf16x8 (&wf)[NFRAG], f32x16 (&acc)[4][RH]) {
    constexpr int NR = RH + 2;
    constexpr int DONE = (P + 1) & 3;
    bf16x8 b[2][NR];
#pragma unroll
    for (int r = 0; r < NR; ++r)
        b[0][r] = *reinterpret_cast<const bf16x8 *>(lbase + (r * LCOLS) * 16);
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        const int kw = gi >> 1, half = gi & 1;
        if (gi + 1 < NG) {
            const int kw2 = (gi + 1) >> 1, half2 = (gi + 1) & 1;
#pragma unroll
            for (int r = 0; r < NR; ++r)
                b[(gi + 1) & 1][r] = *reinterpret_cast<const bf16x8 *>(
                    lbase + half2 * 2 * CH_STRIDE + (r * LCOLS + kw2) * 16);
        }
        // keep the reads of the next group ahead of this group's MFMAs (the scheduler would
        // otherwise sink every read to just before its first use and expose the LDS latency)
        __builtin_amdgcn_sched_barrier(0);
        stage(c, Dp + DIST, gi, lane);
        if (gi < 4) {
            if (EPI) {
                store_unit<RELU, FULL>(c, Dp - 3, acc[DONE], 0, gi);
                store_unit<RELU, FULL>(c, Dp - 3, acc[DONE], 1, gi);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[DONE][gi - 4][i] = HAS_BIAS ? c.bv[HAS_BIAS ? i : 0] : 0.f;
        }
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const int h = r - kh;
                if (h < 0 || h >= RH) continue;
#pragma unroll
                for (int kd = 0; kd < 3; ++kd) {
                    const int slot = (P - kd + 4) & 3;
                    acc[slot][h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        wf[((kd * 3 + kh) * 3 + kw) * 2 + half], b[gi & 1][r], acc[slot][h], 0, 0, 0);
                }
            }
        // weave: after each MFMA let a few of the side-work instructions issue while it executes
#pragma unroll
        for (int i = 0; i < 3 * (RH + 1) * 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x006, 3, 0);   // up to three VALU / SALU
            if (i % 6 == 2) __builtin_amdgcn_sched_group_barrier(0x060, 1, 0);   // a vector memory op
        }
    }
}

template <bool HAS_BIAS, bool RELU>
__global__ __launch_bounds__(kThreads, 1) void conv_mfma_kernel(ConvArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];   // NBUF planes of PLANE_BYTES
    const Geo &g = a.g;
    // Consecutive hardware workgroup ids rotate over the 8 XCDs; give each XCD a contiguous range of
    // logical ids so that patches sharing halo rows/columns meet in the same L2.
    const int per_xcd = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= a.nblocks) return;
    int t = logical;
    const int pw_i = t % a.nw; t /= a.nw;
    const int ph_i = t % a.nh; t /= a.nh;
    const int pd_i = t % a.nd; t /= a.nd;
    const int tile = t;
    const int d0 = pd_i * a.dchunk, h0 = ph_i * PH, w0 = pw_i * PW;      // interior coordinates
    const int dn = min(a.dchunk, g.td - d0);                            // output planes to produce
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hi = lane >> 5;

    // weight fragments: 54 x 16 bytes per lane, resident for the whole march
    bf16x8 wf[NFRAG];
#pragma unroll
    for (int f = 0; f < NFRAG; ++f) {
        const uint4 q = a.wpack[f * 64 + lane];
        wf[f] = *reinterpret_cast<const bf16x8 *>(&q);
    }

    Ctx<HAS_BIAS> c;
    c.plane_elems = static_cast<size_t>(g.ph) * g.pw * C;
    c.tin0 = a.in + static_cast<size_t>(tile) * g.tile_vox * C + d0 * c.plane_elems;
    c.nplanes = dn + 2;
    // Wave w fills chunk plane w (channels 8w..8w+7 of every voxel); load j covers patch-local voxels
    // 64j..64j+63.  Voxels outside the padded tile (ragged patches) are clamped to a valid address;
    // they only feed outputs that are never stored.
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int v = 64 * j + lane;
        const int row = min(h0 + v / LCOLS, g.ph - 1), colv = min(w0 + v % LCOLS, g.pw - 1);
        c.goff[j] = (row * g.pw + colv) * C + wave * 8;
    }
    c.lds_stage = lds + wave * CH_STRIDE;
    c.orow = static_cast<size_t>(g.pw) * C;
    c.obase = a.out + static_cast<size_t>(tile) * g.tile_vox * C +
              ((static_cast<size_t>(d0 + 1) * g.ph + h0 + wave * RH + 1) * g.pw + w0 + col + 1) * C + 4 * hi;
#pragma unroll
    for (int h = 0; h < RH; ++h) c.okrow[h] = h0 + wave * RH + h < g.th && w0 + col < g.tw;
    // the bias is folded into the accumulators: a slot starts from the bias instead of zero
    // (without a bias the slots start from the constant zero and no registers are spent on it)
    if (HAS_BIAS) {
#pragma unroll
        for (int i = 0; i < 16; ++i) c.bv[HAS_BIAS ? i : 0] = a.bias[8 * (i >> 2) + 4 * hi + (i & 3)];
    }
    f32x16 acc[4][RH];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[s][h][i] = HAS_BIAS ? c.bv[HAS_BIAS ? i : 0] : 0.f;

    const char *lbase = lds + lds_off(wave * RH * LCOLS + col, hi);
    const int nplanes = c.nplanes;

    // Prologue: planes 0 .. DIST-1 in flight; plane 0 must have landed before the first MFMA.
#pragma unroll
    for (int i = 0; i < DIST; ++i)
#pragma unroll
        for (int j = 0; j < LOADS; ++j) stage(c, i, j, lane);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // End of a step: plane Dp+1 must be complete before anyone reads it in the next step.  Loads
    // complete in issue order and the only loads issued after plane Dp+1's are those of planes Dp+2 and
    // Dp+3, so "at most 2*LOADS vector memory operations outstanding" implies it is done (stores share
    // the counter and only make the wait more conservative).  A bare s_barrier: __syncthreads() would
    // make the compiler drain every staging load.
#define SP3D_STEP_END()                                                              \
    do {                                                                             \
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DIST - 1) * LOADS) : "memory");    \
        __builtin_amdgcn_s_barrier();                                                \
    } while (0)

    auto march = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        // the first three steps have no finished plane to store (nplanes >= 3 always)
        plane_step<0, false, RELU, FULL>(c, 0, lane, lbase, wf, acc);
        SP3D_STEP_END();
        plane_step<1, false, RELU, FULL>(c, 1, lane, lbase + PLANE_BYTES, wf, acc);
        SP3D_STEP_END();
        plane_step<2, false, RELU, FULL>(c, 2, lane, lbase + 2 * PLANE_BYTES, wf, acc);
        SP3D_STEP_END();
        // steps 3, 4, 5, 6, 7, ...: planes mod 4 = 3, 0, 1, 2, 3, ...
#define SP3D_MAIN_STEP(OFF, PHASE)                                                                   \
    if (D + (OFF) < nplanes) {                                                                       \
        plane_step<PHASE, true, RELU, FULL>(c, D + (OFF), lane, lbase + (PHASE) * PLANE_BYTES, wf, acc); \
        SP3D_STEP_END();                                                                             \
    }
        for (int D = 3; D < nplanes; D += 4) {
            SP3D_MAIN_STEP(0, 3)
            SP3D_MAIN_STEP(1, 0)
            SP3D_MAIN_STEP(2, 1)
            SP3D_MAIN_STEP(3, 2)
        }
#undef SP3D_MAIN_STEP
        // the last output plane (dn-1) finished in the last step; it sits in slot (dn-1) mod 4
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int s = 0; s < 4; ++s)
            if (s == ((dn - 1) & 3)) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    store_unit<RELU, FULL>(c, dn - 1, acc[s], 0, q);
                    store_unit<RELU, FULL>(c, dn - 1, acc[s], 1, q);
                }
            }
    };
    if (h0 + PH <= g.th && w0 + PW <= g.tw) march(std::true_type{});
    else march(std::false_type{});
#undef SP3D_STEP_END
}

}  // namespace

bool conv_mfma_supported(const Geo &g, int ki, int ko, sp_dtype_t dt) {
    return dt == SP_BF16 && ki == C && ko == C && 1LL * g.ph * g.pw * C < 0x7fffffffLL;
}

size_t conv_mfma_ws_bytes(const Geo &, int, int) { return static_cast<size_t>(NFRAG) * 64 * 16; }

int launch_conv_mfma(const void *Pin, const void *w, const float *bias, void *Pout, const Geo &g,
                     int ki, int ko, bool relu, bool dgrad, void *ws, hipStream_t s) {
    (void)ki; (void)ko;
    hipLaunchKernelGGL(pack_weights_kernel, dim3((NFRAG * 64 * 8 + 255) / 256), dim3(256), 0, s,
                       static_cast<const uint16_t *>(w), static_cast<uint16_t *>(ws), dgrad ? 1 : 0);
    int rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    ConvArgs a;
    a.in = static_cast<const uint16_t *>(Pin);
    a.wpack = static_cast<const uint4 *>(ws);
    a.bias = bias;
    a.out = static_cast<uint16_t *>(Pout);
    a.g = g;
    a.nh = (g.th + PH - 1) / PH;
    a.nw = (g.tw + PW - 1) / PW;
    // D chunk: whole tile depth unless that leaves the chip short of workgroups
    long long base = 1LL * g.ntiles * a.nh * a.nw;
    int dchunk = g.td;
    while (base * ((g.td + dchunk - 1) / dchunk) < 1024 && dchunk > 16) dchunk = (dchunk + 1) / 2;
    a.dchunk = dchunk;
    a.nd = (g.td + dchunk - 1) / dchunk;
    const long long nb = base * a.nd;
    if (nb > 0x7ffffff0LL) return SP_EGEOM;
    a.nblocks = static_cast<int>(nb);
    a.relu = relu ? 1 : 0;
    const unsigned grid = static_cast<unsigned>((nb + 7) / 8 * 8);
    // more than 64 KB of dynamic LDS has to be requested explicitly
    using Kern = void (*)(ConvArgs);
    static const Kern kern[2][2] = {{conv_mfma_kernel<false, false>, conv_mfma_kernel<false, true>},
                                    {conv_mfma_kernel<true, false>, conv_mfma_kernel<true, true>}};
    static const hipError_t attr = [] {
        for (int i = 0; i < 4; ++i) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern[i >> 1][i & 1]),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }();
    if (attr != hipSuccess) return record_hip(attr);
    hipLaunchKernelGGL(kern[bias ? 1 : 0][relu ? 1 : 0], dim3(grid), dim3(kThreads), LDS_BYTES, s, a);
    return record_hip(hipGetLastError());
}

}  // namespace sp3d
