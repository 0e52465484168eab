// bf16 3x3 (2-D variant, geometry flag `flat`) and 3x3x3 convolution for wide layers on few voxels - the bottom
// levels of the 2-D U-Net (Sec. 3: 512 and 1024 filters on tiles of 16 x 16 voxels and less) and the 16^3 level of
// the 3-D one - as an output-stationary implicit GEMM on the gfx950 matrix cores.  Serves conv3d_fwd and, on weights packed with
// mirrored taps and swapped channel roles, conv3d_dgrad, like the plane-marching kernels of conv_mfma.hip.
//
// Why a second kernel family.  The marching kernels keep the weights of ONE pair of input chunks in
// registers and stream voxels past them; a layer with 1024 input channels is 16 launches that hand fp32
// partial sums to each other through memory, and on tiles of 8 x 8 voxels each launch is a march of a few
// steps in a mostly empty patch.  Here the roles are swapped: a workgroup owns 256 output voxels x 128 output
// channels, keeps their sums in registers (8 accumulators of 32 x 32 per wave) over ALL taps and input
// channels, and streams the weights: one launch per layer, no partial sums, and voxels are numbered across
// rows, slices and tiles, so every MFMA column is a real voxel whatever the tile shape.  (With the 3x3x3 kernel
// the marching kernels do three times the MFMAs per staged byte; they are level with this family at 32^3 voxels
// and ahead beyond, so in 3-D it serves the smallest level only: see conv_gemm_preferred.)
//
// Operands (v_mfma_f32_32x32x16_bf16, A = weights [32 output channels][16 input channels], B = voxels
// [16 input channels][32 voxels]).  B: lane l supplies voxel l % 32, channels 8 (l / 32) .. + 7 of the
// 16-channel half: 16 contiguous bytes of the NDHWC record of the voxel one tap away, one global load per
// lane and fragment, no LDS (the taps of a kernel row re-read the same records from the vector cache).
// A: the packed fragments of conv_mfma.hip (1 KB each, lane-major), shared by the four waves of a workgroup
// through LDS: a K step is one 32-channel input chunk x one kernel row (kw = 0, 1, 2): 24 fragments for the
// workgroup's 4 output blocks, double buffered; they and the B fragments of a step are fetched two steps
// ahead; one barrier per step (48 MFMAs per wave).
//
// Output box growth, two input tensors (concatenation without a copy), two output tensors, bias, ReLU and the
// ReLU mask of the data gradient behave as in conv_mfma.hip.  The order of the additions is fixed (kernel rows,
// then chunks, then taps), so results are reproducible and do not depend on the voxel's position.
#include "common.h"

namespace sp3d {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// (a plain vector type: arrays of the runtime's uint4 class stayed in scratch memory - 12 stores and 12 loads per
// K step, each with a wait that drained the voxel-fragment loads in flight)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int C = 32;                            // channels of a chunk / block
constexpr int CB = 4;                            // output blocks per workgroup
constexpr int VBMAX = 2;                         // 32-voxel segments per wave: 2, or 1 for layers that would
                                                 // otherwise leave half of the compute units without a workgroup
constexpr int kWaves = 4, kThreads = 256;
constexpr int wg_vox(int vb) { return kWaves * vb * 32; }      // 256 (or 128) output voxels per workgroup
constexpr int ROW = 3;                           // taps per K step (one row of the kernel)
constexpr int STAGE_FRAGS = CB * ROW * 2;        // 24 weight fragments (1 KB each) per K step
constexpr int STAGE_U4 = STAGE_FRAGS * 64;       // in 16-byte pieces: 6 per thread
constexpr int STAGE_LOADS = STAGE_U4 / kThreads;
constexpr int STAGE_BYTES = STAGE_FRAGS * 1024;
constexpr int LDS_BYTES = 2 * STAGE_BYTES;       // 49152
constexpr int NTAP_PACK = 27;                    // packed weights: 27 tap slots per (chunk, block); the 3x3 kernel of the
                                                 // 2-D variant sits in 9 .. 17 (the taps with kd = 1)
// kernel rows (kd, kh) of a K loop: 3 in the 2-D variant (KD = 1), 9 in 3-D (KD = 3)
constexpr int nrows(int KD) { return 3 * KD; }

enum Epilogue { kNone = 0, kRelu = 1, kMask = 2 };

struct GemmArgs {
    const uint16_t *in;      // input channels [0, in_ca): in_cs channels per voxel
    const uint16_t *in2;     // input channels [in_ca, ki): in2_cs channels per voxel (NULL: one tensor)
    int in_cs, in2_cs, in_ca;
    const uint4 *wpack;      // [nci][nco][27][2][64] x 16 bytes
    const float *bias;       // bias of all output channels or NULL
    uint16_t *out;           // output channels [0, out_ca): out_cs channels per voxel
    uint16_t *out2;          // output channels [out_ca, ko): out2_cs per voxel (NULL: one tensor)
    int out_cs, out2_cs, out_ca;
    const uint16_t *mask;    // kMask: tensor laid out like `out`; results are zeroed where it is not positive
    Geo g;
    int nci, nco;            // input chunks, output blocks
    int nvg;                 // voxel groups of wg_vox(VB)
    int nblocks;             // nvg * nco / CB real workgroups (grid is rounded up to a multiple of 8)
    int nvox;                // ntiles * ed * eh * ew: voxels of the largest output box, every tile
    int ed, eh, ew;          // largest output box of the grid (interior grown on both sides)
    FastDiv dbox, dplane, drow;      // ed * eh * ew, eh * ew, ew
};

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    union { bf16x2 v; uint32_t u; } r;
    r.v = __builtin_convertvector(f32x2{a, b}, bf16x2);
    return r.u;
}

// two bf16 in a word -> 0xffff in each half whose value is positive (not zero, not negative, not NaN)
__device__ __forceinline__ uint32_t positive_halves(uint32_t v) {
    const uint32_t lo = v & 0xffffu, hi = v >> 16;
    return ((lo - 1u) < 0x7f80u ? 0x0000ffffu : 0u) | ((hi - 1u) < 0x7f80u ? 0xffff0000u : 0u);
}

// Per-thread state of the K loop.
struct Ctx {
    long long pv[VBMAX];         // padded voxel index of this lane's output voxel in segment s
    int hi;                      // lane / 32: which 8 channels of a 16-channel half this lane supplies
    int tid;
    int cg;                      // first output block of the workgroup / CB
    long long plane, row;        // voxel strides of the padded tile
};

// Source of input chunk i: tensor, channels per voxel, channel offset.
struct InSrc { const uint16_t *base; int cs, co; };
__device__ __forceinline__ InSrc in_src(const GemmArgs &a, int i) {
    const int c0 = C * i;
    if (a.in2 && c0 >= a.in_ca) return InSrc{a.in2, a.in2_cs, c0 - a.in_ca};
    return InSrc{a.in, a.in_cs, c0};
}

// Voxel offset of kernel row r (= kh in the 2-D variant, 3 kd + kh in 3-D) at kw = 0, relative to the output voxel.
template <int KD>
__device__ __forceinline__ long long row_offset(const Ctx &c, int r) {
    if (KD == 1) return (r - 1) * c.row - 1;
    const int kd = r / 3, kh = r - 3 * kd;
    return (kd - 1) * c.plane + (kh - 1) * c.row - 1;
}

// next K step, clamped to the last one.  Kernel rows outermost, chunks inside: a voxel's record of two
// neighbouring chunks is one 128-byte line, so the second chunk finds in the vector cache what the first fetched
template <int KD>
__device__ __forceinline__ void advance(const GemmArgs &a, int &i, int &r) {
    int ni = i + 1, nr = r;
    if (ni == a.nci) { ni = 0; ++nr; }
    if (nr < nrows(KD)) { i = ni; r = nr; }
}

// Issue the loads of K step (chunk i, row r): this thread's share of the 24 weight fragments (to registers, on
// their way to LDS) and this lane's B fragments of the step.
template <int VB, int KD>
__device__ __forceinline__ void fetch(const GemmArgs &a, const Ctx &c, int i, int r, u32x4 (&areg)[STAGE_LOADS],
                                      bf16x8 (&b)[VB][ROW][2]) {
    const int tap0 = (KD == 1 ? 9 : 0) + ROW * r;
#pragma unroll
    for (int j = 0; j < STAGE_LOADS; ++j) {
        const int e = j * kThreads + c.tid;                     // piece of the stage
        const int cb = e / (ROW * 2 * 64), x = e - cb * (ROW * 2 * 64);
        const size_t frag0 = (static_cast<size_t>(i * a.nco + c.cg * CB + cb) * NTAP_PACK + tap0) * 2;
        areg[j] = reinterpret_cast<const u32x4 *>(a.wpack)[frag0 * 64 + x];
    }
    const InSrc src = in_src(a, i);
    const long long ro = row_offset<KD>(c, r);
#pragma unroll
    for (int s = 0; s < VB; ++s) {
        const uint16_t *p = src.base + (c.pv[s] + ro) * src.cs + src.co + 8 * c.hi;
#pragma unroll
        for (int kw = 0; kw < ROW; ++kw)
#pragma unroll
            for (int half = 0; half < 2; ++half)
                b[s][kw][half] = *reinterpret_cast<const bf16x8 *>(p + static_cast<long long>(kw) * src.cs + 16 * half);
    }
}

// All MFMAs of one K step: weights from LDS stage `abuf`, voxels from registers.
template <int VB>
__device__ __forceinline__ void contract(const char *abuf, int lane, const bf16x8 (&b)[VB][ROW][2],
                                         f32x16 (&acc)[CB][VB]) {
#pragma unroll
    for (int kw = 0; kw < ROW; ++kw)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            bf16x8 w[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
                w[cb] = *reinterpret_cast<const bf16x8 *>(abuf + ((cb * ROW + kw) * 2 + half) * 1024 + lane * 16);
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int s = 0; s < VB; ++s)
                    acc[cb][s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[cb], b[s][kw][half], acc[cb][s], 0, 0, 0);
        }
}

// K step j on LDS stage j % 2 with the voxel fragments `bc`.  The loads of step j + 2 are issued here (voxel
// fragments into `bn`, this thread's share of the weight fragments into `an`) and have a whole step to arrive:
// the compiler is free to place them anywhere between the two barriers.  The weights of step j + 1, loaded during
// step j - 1 into `aw`, go to the other LDS stage, which every wave left at the barrier that ended step j - 1.
// (i, r) = chunk and kernel row of step j + 2; past the last step it stays there: those loads are harmless,
// and what they fill is never read.
template <int VB, int KD>
__device__ __forceinline__ void step(const GemmArgs &a, const Ctx &c, char *cur, char *other, int lane, int &i, int &r,
                                     const bf16x8 (&bc)[VB][ROW][2], bf16x8 (&bn)[VB][ROW][2],
                                     const u32x4 (&aw)[STAGE_LOADS], u32x4 (&an)[STAGE_LOADS], f32x16 (&acc)[CB][VB]) {
    fetch<VB, KD>(a, c, i, r, an, bn);
    contract(cur, lane, bc, acc);
    u32x4 *dst = reinterpret_cast<u32x4 *>(other);
#pragma unroll
    for (int j = 0; j < STAGE_LOADS; ++j) dst[j * kThreads + c.tid] = aw[j];
    __syncthreads();
    advance<KD>(a, i, r);
}

template <int RELU, bool HAS_BIAS, int VB, int KD>
__global__ __launch_bounds__(kThreads, 1) void conv_gemm_kernel(GemmArgs a) {
    extern __shared__ __align__(16) char lds[];
    // workgroups of one XCD (blockIdx % 8) get consecutive logical ids: they share output blocks, i.e. weights
    const int per_xcd = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= a.nblocks) return;
    const Geo &g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    Ctx c;
    c.tid = tid;
    c.hi = lane >> 5;
    c.cg = logical / a.nvg;
    const int vg = logical - c.cg * a.nvg;
    c.row = g.pw;
    c.plane = static_cast<long long>(g.ph) * g.pw;

    // this lane's output voxels: index q over (tile, d, h, w) of the largest output box; a tile whose own box is
    // smaller (no neighbour on that side) computes nothing for the voxels outside it
    bool ok[VB];
#pragma unroll
    for (int s = 0; s < VB; ++s) {
        const long long q = (static_cast<long long>(vg * kWaves + wave) * VB + s) * 32 + (lane & 31);
        const bool in = q < a.nvox;
        const uint32_t qq = in ? static_cast<uint32_t>(q) : 0u;
        const uint32_t tile = fdiv(qq, a.dbox), rb = fmod_(qq, tile, a.dbox);
        uint32_t d = fdiv(rb, a.dplane);
        const uint32_t rp = fmod_(rb, d, a.dplane);
        uint32_t h = fdiv(rp, a.drow), w = fmod_(rp, h, a.drow);
        const TileBox bx = tile_box(g, static_cast<int>(tile));
        ok[s] = in && static_cast<int>(d) < bx.bd && static_cast<int>(h) < bx.bh && static_cast<int>(w) < bx.bw;
        if (!ok[s]) d = h = w = 0;            // a voxel that exists: its loads stay inside the tile, its result is dropped
        c.pv[s] = static_cast<long long>(tile) * g.tile_vox + bx.org + (d + 1) * c.plane + (h + 1) * c.row + (w + 1);
    }

    // accumulators start from the bias: lane l holds channels 8 (e / 4) + 4 (l / 32) + e % 4 of a block
    f32x16 acc[CB][VB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        f32x16 v;
#pragma unroll
        for (int e = 0; e < 16; ++e)
            v[e] = HAS_BIAS ? a.bias[C * (c.cg * CB + cb) + 8 * (e >> 2) + 4 * c.hi + (e & 3)] : 0.f;
#pragma unroll
        for (int s = 0; s < VB; ++s) acc[cb][s] = v;
    }

    // K loop: 3 kernel rows x nci chunks.  Loads run two steps ahead of the MFMAs that use them, so the
    // voxel fragments rotate through three register sets and the weight pieces through two; six steps per
    // iteration keep every set a compile-time name (the step count is a multiple of 6: nci is even).
    bf16x8 b0[VB][ROW][2], b1[VB][ROW][2], b2[VB][ROW][2];
    u32x4 a0[STAGE_LOADS], a1[STAGE_LOADS];
    char *const s0 = lds, *const s1 = lds + STAGE_BYTES;
    int i = 0, r = 0;
    fetch<VB, KD>(a, c, i, r, a0, b0);
    advance<KD>(a, i, r);
    {
        u32x4 *dst = reinterpret_cast<u32x4 *>(s0);
#pragma unroll
        for (int j = 0; j < STAGE_LOADS; ++j) dst[j * kThreads + tid] = a0[j];
    }
    fetch<VB, KD>(a, c, i, r, a1, b1);
    advance<KD>(a, i, r);
    __syncthreads();
    const int nk = a.nci * nrows(KD);
    for (int k = 0; k < nk; k += 6) {
        step<VB, KD>(a, c, s0, s1, lane, i, r, b0, b2, a1, a0, acc);
        step<VB, KD>(a, c, s1, s0, lane, i, r, b1, b0, a0, a1, acc);
        step<VB, KD>(a, c, s0, s1, lane, i, r, b2, b1, a1, a0, acc);
        step<VB, KD>(a, c, s1, s0, lane, i, r, b0, b2, a0, a1, acc);
        step<VB, KD>(a, c, s0, s1, lane, i, r, b1, b0, a1, a0, acc);
        step<VB, KD>(a, c, s1, s0, lane, i, r, b2, b1, a0, a1, acc);
    }

    // epilogue: ReLU / mask, convert, 8-byte stores (4 channels of a voxel)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const int co = C * (c.cg * CB + cb);
        uint16_t *obase = a.out;
        int ocs = a.out_cs, oco = co;
        if (a.out2 && co >= a.out_ca) { obase = a.out2; ocs = a.out2_cs; oco = co - a.out_ca; }
#pragma unroll
        for (int s = 0; s < VB; ++s) {
            if (!ok[s]) continue;
            uint16_t *o = obase + c.pv[s] * ocs + oco + 4 * c.hi;
            const uint16_t *m = RELU == kMask ? a.mask + c.pv[s] * a.out_cs + co + 4 * c.hi : nullptr;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v0 = acc[cb][s][4 * q], v1 = acc[cb][s][4 * q + 1], v2 = acc[cb][s][4 * q + 2], v3 = acc[cb][s][4 * q + 3];
                if (RELU == kRelu) {
                    v0 = v0 < 0.f ? 0.f : v0; v1 = v1 < 0.f ? 0.f : v1;
                    v2 = v2 < 0.f ? 0.f : v2; v3 = v3 < 0.f ? 0.f : v3;
                }
                uint2 pk = make_uint2(pack2(v0, v1), pack2(v2, v3));
                if (RELU == kMask) {
                    const uint2 mv = *reinterpret_cast<const uint2 *>(m + 8 * q);
                    pk.x &= positive_halves(mv.x);
                    pk.y &= positive_halves(mv.y);
                }
                *reinterpret_cast<uint2 *>(o + 8 * q) = pk;
            }
        }
    }
}

// largest output box of the grid
struct Box { int ed, eh, ew; };
Box max_box(const Geo &g) { return Box{g.td + 2 * grow_d(g), g.th + 2 * g.grow, g.tw + 2 * g.grow}; }

}  // namespace

// Layers this family takes over from the plane-marching kernels.  2-D variant (measured on 16 slices; marching ->
// here, before this kernel's weight pieces left scratch memory): 512 channels on 32 x 32 voxels 0.37 -> 0.21 ms, 1024
// on 32 x 32 1.30 -> 0.70 ms, 1024 on 16 x 16 0.48 -> 0.37 ms; at 256 channels the marching kernels are as fast.  3-D:
// the bottom level of a deep network only - 1024 channels on 16^3 voxels 0.80 -> 0.40 ms on a 2 x 2 x 1 grid and 1.01 ->
// 0.39 ms on 4 x 4 x 1 (tiles of 4 x 4 x 16 voxels leave most of a marching patch empty; here every MFMA column is a real
// voxel), 512 -> 1024 0.37 -> 0.19 ms; on 32^3 voxels (512 channels) the two families are level (0.55 - 0.64 ms either way)
// and on 64^3 the marching kernels win, because a staged plane feeds 27 taps there and 9 here.  The criterion looks
// at the tile interiors only, so a layer is served by the same family whatever its output box growth.
bool conv_gemm_preferred(const Geo &g, int ki, int ko) {
    const long long nint = 1LL * g.ntiles * g.int_vox;
    const Box b = max_box(g);
    const long long nbox = 1LL * g.ntiles * b.ed * b.eh * b.ew;
    if (ki < 512 || ki % (2 * C) != 0 || ko % (C * CB) != 0 || nbox >= (1LL << 30)) return false;
    return nint <= (g.flat ? (1 << 16) : (1 << 13));
}

// wpack: the layer's weights in the fragment order of conv_mfma.hip (already packed, in the workspace).
int launch_conv_gemm(const void *Pin, const void *wpack, const float *bias, void *Pout, const Geo &g, int ki, int ko,
                     bool relu, hipStream_t s, const void *mask, const ConvSplit *split) {
    GemmArgs a;
    a.in = static_cast<const uint16_t *>(Pin);
    a.in2 = nullptr;
    a.in_cs = ki;
    a.in2_cs = 0;
    a.in_ca = ki;
    if (split && split->in2) {
        a.in2 = static_cast<const uint16_t *>(split->in2);
        a.in_ca = split->in_ca;
        a.in_cs = split->in_ca;
        a.in2_cs = ki - split->in_ca;
    }
    a.out = static_cast<uint16_t *>(Pout);
    a.out2 = nullptr;
    a.out_cs = ko;
    a.out2_cs = 0;
    a.out_ca = ko;
    if (split && split->out2) {
        a.out2 = static_cast<uint16_t *>(split->out2);
        a.out_ca = split->out_ca;
        a.out_cs = split->out_ca;
        a.out2_cs = ko - split->out_ca;
    }
    a.wpack = static_cast<const uint4 *>(wpack);
    a.bias = bias;
    a.mask = static_cast<const uint16_t *>(mask);
    a.g = g;
    a.nci = ki / C;
    a.nco = ko / C;
    const Box b = max_box(g);
    a.ed = b.ed;
    a.eh = b.eh;
    a.ew = b.ew;
    a.nvox = static_cast<int>(1LL * g.ntiles * b.ed * b.eh * b.ew);
    a.dbox = make_fastdiv(static_cast<uint32_t>(b.ed * b.eh * b.ew));
    a.dplane = make_fastdiv(static_cast<uint32_t>(b.eh * b.ew));
    a.drow = make_fastdiv(static_cast<uint32_t>(b.ew));
    // 256 voxels per workgroup; 128 where that leaves at most half of the 256 compute units with a workgroup (the
    // kernel is bound by its voxel-fragment loads, which then spread over twice the vector caches)
    const int nvg2 = (a.nvox + wg_vox(2) - 1) / wg_vox(2);
    const int vb = nvg2 * (a.nco / CB) <= 128 ? 1 : 2;
    a.nvg = (a.nvox + wg_vox(vb) - 1) / wg_vox(vb);
    a.nblocks = a.nvg * (a.nco / CB);
    const unsigned grid = static_cast<unsigned>((a.nblocks + 7) / 8 * 8);
    using Kern = void (*)(GemmArgs);
    // [3-D][segments per wave - 1][bias][epilogue]; a bias never comes with a mask
#define SP3D_GEMM_TABLE(KD)                                                                                             \
    {{{conv_gemm_kernel<kNone, false, 1, KD>, conv_gemm_kernel<kRelu, false, 1, KD>, conv_gemm_kernel<kMask, false, 1, KD>},  \
      {conv_gemm_kernel<kNone, true, 1, KD>, conv_gemm_kernel<kRelu, true, 1, KD>, conv_gemm_kernel<kMask, false, 1, KD>}},   \
     {{conv_gemm_kernel<kNone, false, 2, KD>, conv_gemm_kernel<kRelu, false, 2, KD>, conv_gemm_kernel<kMask, false, 2, KD>},  \
      {conv_gemm_kernel<kNone, true, 2, KD>, conv_gemm_kernel<kRelu, true, 2, KD>, conv_gemm_kernel<kMask, false, 2, KD>}}}
    static const Kern kern[2][2][2][3] = {SP3D_GEMM_TABLE(1), SP3D_GEMM_TABLE(3)};
#undef SP3D_GEMM_TABLE
    const int epi = mask ? kMask : (relu ? kRelu : kNone);
    hipLaunchKernelGGL(kern[g.flat ? 0 : 1][vb - 1][bias ? 1 : 0][epi], dim3(grid), dim3(kThreads), LDS_BYTES, s, a);
    return record_hip(hipGetLastError());
}

}  // namespace sp3d
