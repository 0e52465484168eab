// bf16 implicit-GEMM 3x3x3 convolution on padded tiles for Cin = Cout = 32, on the gfx950 matrix
// cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).  Serves conv3d_fwd and, with mirrored taps
// and swapped channel roles, conv3d_dgrad.
//
// Work decomposition.  A workgroup (4 waves) owns an output patch of 8 rows (H) x 32 columns (W)
// of one tile and marches along D.  Each input plane (10 x 34 voxels x 32 channels, 21.25 KB) is
// staged once in LDS (double buffered: the next plane is fetched from HBM into registers while the
// current one is consumed).  A wave owns 2 of the 8 rows and keeps the accumulators of THREE
// consecutive output planes in registers: input plane D feeds output planes D, D-1, D-2 through
// taps kd = 0, 1, 2, so an input fragment read from LDS once is used by up to 3 (kd) x 2 (kh)
// MFMAs.  All 27 x 2 weight fragments (32 x 16 each) live in registers for the whole march.
//
// MFMA operand roles: A = weights [M = Cout][K = 16 input channels], B = voxels [K][N = 32 voxels
// along W], D[M = Cout][N = voxel].  Lane l of B supplies voxel l%32, channels 8*(l/32)..+7 of the
// 16-channel half; lane l of D holds voxel l%32, channels 8*(i/4) + 4*(l/32) + i%4 for i = 0..15.
#include "common.h"

namespace sp3d {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int C = 32;                       // channels in and out
constexpr int kWaves = 4, kThreads = 256;
constexpr int RH = 2;                       // output rows per wave
constexpr int PH = RH * kWaves;             // patch rows
constexpr int PW = 32;                      // patch columns = MFMA N
constexpr int LROWS = PH + 2, LCOLS = PW + 2;
constexpr int PLANE_VOX = LROWS * LCOLS;    // 340
constexpr int PLANE_CHUNKS = PLANE_VOX * 4; // 16-byte chunks per plane
constexpr int ROW_CHUNKS = LCOLS * 4;       // 136
constexpr int LOADS = (PLANE_CHUNKS + kThreads - 1) / kThreads;   // 6
constexpr int NFRAG = 27 * 2;               // weight fragments per lane (16 bytes each)

// Byte offset of 16-byte chunk c (0..3) of voxel v in a staged plane.  The chunk index is XORed
// with bits 1..2 of the voxel index so that 8 consecutive voxels at the same logical chunk fall
// into 8 different 16-byte bank groups (a voxel record is 64 bytes = half of the 128-byte bank row).
__device__ __forceinline__ int lds_off(int v, int c) { return v * 64 + ((c ^ ((v >> 1) & 3)) << 4); }

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

template <int P>   // P = (input plane index) mod 3
__device__ __forceinline__ void plane_step(const char *lds, const bf16x8 (&wf)[NFRAG],
                                           f32x16 (&acc)[3][RH], int wave, int lane) {
    const int col = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int r = 0; r < RH + 2; ++r) {
                const int v = (wave * RH + r) * LCOLS + col + kw;
                const bf16x8 b = *reinterpret_cast<const bf16x8 *>(lds + lds_off(v, 2 * half + hi));
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) {
                    const int h = r - kh;
                    if (h < 0 || h >= RH) continue;
#pragma unroll
                    for (int kd = 0; kd < 3; ++kd) {
                        const int slot = (P - kd + 3) % 3;
                        acc[slot][h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            wf[((kd * 3 + kh) * 3 + kw) * 2 + half], b, acc[slot][h], 0, 0, 0);
                    }
                }
            }
}

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    return static_cast<uint32_t>(f32_to_bf16(a)) | (static_cast<uint32_t>(f32_to_bf16(b)) << 16);
}

__global__ __launch_bounds__(kThreads, 1) void conv_mfma_kernel(ConvArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];   // 2 planes of PLANE_VOX * 64 bytes
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
    const uint16_t *tin = a.in + static_cast<size_t>(tile) * g.tile_vox * C;
    uint16_t *tout = a.out + static_cast<size_t>(tile) * g.tile_vox * C;

    // weight fragments: 54 x 16 bytes per lane, resident for the whole march
    bf16x8 wf[NFRAG];
#pragma unroll
    for (int f = 0; f < NFRAG; ++f) {
        const uint4 q = a.wpack[f * 64 + lane];
        wf[f] = *reinterpret_cast<const bf16x8 *>(&q);
    }

    // staging: this thread's chunks of a plane.  Patch-local (row, col) -> padded tile (h0+row, w0+col);
    // chunks outside the padded tile (ragged patches) are staged as zeros.
    int src_off[LOADS], dst_off[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int q = tid + i * kThreads;
        const int row = q / ROW_CHUNKS, rem = q % ROW_CHUNKS, colv = rem >> 2, c = rem & 3;
        const bool ok = q < PLANE_CHUNKS && h0 + row < g.ph && w0 + colv < g.pw;
        src_off[i] = ok ? ((h0 + row) * g.pw + w0 + colv) * C + c * 8 : -1;
        dst_off[i] = q < PLANE_CHUNKS ? lds_off(row * LCOLS + colv, c) : -1;
    }
    const size_t plane_elems = static_cast<size_t>(g.ph) * g.pw * C;
    uint4 stage[LOADS];
    auto fetch = [&](int dplane) {   // padded plane index d0 + dplane
        const uint16_t *p = tin + (d0 + dplane) * plane_elems;
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            stage[i] = src_off[i] >= 0 ? *reinterpret_cast<const uint4 *>(p + src_off[i])
                                       : make_uint4(0, 0, 0, 0);
    };
    auto commit = [&](int buf) {
        char *base = lds + buf * (PLANE_VOX * 64);
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            if (dst_off[i] >= 0) *reinterpret_cast<uint4 *>(base + dst_off[i]) = stage[i];
    };

    f32x16 acc[3][RH];
#pragma unroll
    for (int s = 0; s < 3; ++s)
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[s][h][i] = 0.f;

    const int col = lane & 31, hi = lane >> 5;
    float bv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) bv[i] = a.bias ? a.bias[8 * (i >> 2) + 4 * hi + (i & 3)] : 0.f;

    // Finish output plane d (local index) held in `slot`: bias, ReLU, bf16, store, clear.
    auto finish = [&](int d, f32x16 (&s)[RH]) {
        if (d >= 0 && d < dn) {
#pragma unroll
            for (int h = 0; h < RH; ++h) {
                const int oh = h0 + wave * RH + h, ow = w0 + col;
                if (oh < g.th && ow < g.tw) {
                    uint16_t *o = tout + ((static_cast<size_t>(d0 + d + 1) * g.ph + oh + 1) * g.pw + ow + 1) * C +
                                  4 * hi;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float v0 = s[h][4 * q] + bv[4 * q], v1 = s[h][4 * q + 1] + bv[4 * q + 1];
                        float v2 = s[h][4 * q + 2] + bv[4 * q + 2], v3 = s[h][4 * q + 3] + bv[4 * q + 3];
                        if (a.relu) {
                            v0 = v0 > 0.f ? v0 : 0.f; v1 = v1 > 0.f ? v1 : 0.f;
                            v2 = v2 > 0.f ? v2 : 0.f; v3 = v3 > 0.f ? v3 : 0.f;
                        }
                        *reinterpret_cast<uint2 *>(o + 8 * q) = make_uint2(pack2(v0, v1), pack2(v2, v3));
                    }
                }
            }
        }
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int i = 0; i < 16; ++i) s[h][i] = 0.f;
    };

    // prologue: plane 0 into buffer 0
    fetch(0);
    commit(0);
    __syncthreads();

    const int nplanes = dn + 2;
    for (int D = 0; D < nplanes; D += 3) {
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const int Dp = D + p;
            if (Dp < nplanes) {
                const int buf = Dp & 1;
                if (Dp + 1 < nplanes) fetch(Dp + 1);
                const char *cur = lds + buf * (PLANE_VOX * 64);
                if (p == 0) plane_step<0>(cur, wf, acc, wave, lane);
                else if (p == 1) plane_step<1>(cur, wf, acc, wave, lane);
                else plane_step<2>(cur, wf, acc, wave, lane);
                if (Dp + 1 < nplanes) commit(buf ^ 1);
                __syncthreads();
                // output plane Dp-2 has now received all three kd contributions
                finish(Dp - 2, acc[(p + 1) % 3]);
            }
        }
    }
}

}  // namespace

bool conv_mfma_supported(const Geo &g, int ki, int ko, sp_dtype_t dt) {
    (void)g;
    return dt == SP_BF16 && ki == C && ko == C;
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
    hipLaunchKernelGGL(conv_mfma_kernel, dim3(grid), dim3(kThreads), 2 * PLANE_VOX * 64, s, a);
    return record_hip(hipGetLastError());
}

}  // namespace sp3d
