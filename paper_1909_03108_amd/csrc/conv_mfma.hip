// bf16 implicit-GEMM 3x3x3 convolution on padded tiles for channel counts that are multiples of 32,
// on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).  Serves conv3d_fwd and,
// with mirrored taps and swapped channel roles, conv3d_dgrad.
//
// The kernel proper contracts ONE 32-channel input chunk into one 32-channel output block.  Wider
// layers run it once per input chunk (one launch each, every output block in the same launch): the
// first chunk writes fp32 partial sums to the workspace, later chunks add to them, the last one adds,
// applies ReLU and stores bf16.  The order of the additions is fixed, so results are reproducible.
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
// 2-D variant (template parameter KD = 1; geometry flag `flat`): the kernel has extent 1 along D, so a staged
// plane feeds only its own output plane (tap kd = 1 of the scheme above; the MFMAs of kd = 0, 2 and their
// weight fragments are left out).  The march, the ring and the epilogue timing are unchanged.
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

// How a launch treats the fp32 partial sums of a layer with several input chunks.
enum Mode { kSingle = 0,   // only chunk: bias, ReLU, store bf16
            kFirst = 1,    // first chunk: bias, store fp32 partial
            kMiddle = 2,   // add partial, store fp32 partial
            kLast = 3 };   // add partial, ReLU, store bf16

struct ConvArgs {
    const uint16_t *in;     // input tensor; this launch reads channels [in_co, in_co + 32) of in_cs
    const uint16_t *in2;    // pair kernel: tensor, channels per voxel and offset of the pair's second chunk
    int in2_cs, in2_co;     //   (the same tensor 32 channels further on, or a second input tensor)
    const uint4 *wpack;     // fragments of this input chunk: [nco][27][2][64] x 16 bytes
    const float *bias;      // bias of all output channels or NULL
    uint16_t *out;          // output tensor (out_cs channels per voxel)
    uint16_t *out2;         // optional second output tensor (out2_cs channels per voxel): output channels
    int out_ca, out2_cs;    //   [out_ca, ko) go there, [0, out_ca) to `out`
    const uint16_t *mask;   // kMask: tensor laid out like `out`; results are zeroed where it is not positive
    uint16_t *bits;         // kMaskBits (read) / kReluBits (written): one bit per output value, see relu_bit
    float *part;            // fp32 partial sums in fragment order (see part_unit)
    Geo g;
    int in_cs, in_co, out_cs;
    int nco;                // output blocks of 32 channels (all handled by this launch)
    int dchunk;             // output planes per workgroup
    int nd, nh, nw;         // patches per tile along D, H, W
    int nblocks;            // real workgroups (grid is rounded up to a multiple of 8)
    int fold, fold_w;       // 2-D variant, tiles narrower than half a patch: `fold` consecutive slices lie side by
                            // side in a patch, each in a strip of fold_w = box width + 2 columns (fold = 1: none)
    int gather;             // 1: margin voxels that have a neighbour tile are staged from that tile's interior
};

// Gathered halos (SP_HALO_GATHER).  The voxel that the exchange would copy into a tile's margin lies, in the
// neighbour tile, exactly one tile extent further along the axis: margin row 0 of tile (a, b, c) is interior row
// th of tile (a, b - 1, c).  A staging load that falls into a margin therefore only needs a constant added to its
// source offset - tile stride of the neighbour minus the tile extent along the axis - and the exchange is not
// needed at all.  Along H and W the constant is per lane and fixed for the whole march (it goes into goff);
// along D it applies to the first and the last staged plane of a march that starts / ends at the tile's own
// first / last plane (dlo, dhi: wave-uniform).  The offsets of several axes add up (edges, corners).  Margins
// at the volume border are still read from the tensor itself, where they hold the zero padding.
struct GatherShift {
    int hm, hp, wm, wp;         // element offsets for margin row 0 / th + 1 and margin column 0 / tw + 1 (0: no neighbour)
    ptrdiff_t dm, dp;           // element offsets for margin plane 0 / td + 1
};
__device__ __forceinline__ GatherShift gather_shift(const Geo &g, int tile, int cs) {
    GatherShift s;
    const int tc = tile % g.gw, t1 = tile / g.gw;
    const int tb = t1 % g.gh, ta = (t1 / g.gh) % g.gd;
    const ptrdiff_t tv = static_cast<ptrdiff_t>(g.tile_vox);
    const ptrdiff_t w = (tv - g.tw) * cs;                                              // to tile c + 1
    const ptrdiff_t h = (tv * g.gw - static_cast<ptrdiff_t>(g.th) * g.pw) * cs;         // to tile b + 1
    const ptrdiff_t d = (tv * g.gw * g.gh - static_cast<ptrdiff_t>(g.td) * g.ph * g.pw) * cs;   // to tile a + 1
    s.wm = tc > 0 ? static_cast<int>(-w) : 0;
    s.wp = tc < g.gw - 1 ? static_cast<int>(w) : 0;
    s.hm = tb > 0 ? static_cast<int>(-h) : 0;
    s.hp = tb < g.gh - 1 ? static_cast<int>(h) : 0;
    s.dm = ta > 0 ? -d : 0;
    s.dp = ta < g.gd - 1 ? d : 0;
    return s;
}

// Slices side by side (2-D variant).  A tile of 8 x 8 voxels fills a quarter of the 32 columns that the MFMAs of a
// patch compute.  Slices do not interact, so `fold` of them share a patch: strip s of the staged plane holds
// columns 0 .. box width + 1 of slice s, and a plane step handles `fold` slices at once (output columns whose
// 3-column window straddles two strips are computed and dropped).  Only per-lane offsets change: the source
// offsets of the staging loads, the output / mask position of a lane, and the strides of a step; the kernels'
// marches are untouched.  Staged "plane" G then means slices F (G - 1) + 1 + s of the chunk (in padded
// coordinates), so that plane G still feeds output step G - 1; planes 0 and the last, which feed no output,
// are clamped to their neighbours instead of reaching outside the tile.
struct FoldCol { int s, c; };      // strip and column inside it
__device__ __forceinline__ FoldCol fold_col(int col, int fold, int fold_w) {
    if (fold == 1) return FoldCol{0, col};
    const int s = col / fold_w;
    return FoldCol{s, col - s * fold_w};
}

// Pre-swizzle the weights into MFMA A-fragment order.  wpack[chunk i][block j][tap][half][lane] = the 8
// input channels k = 32i + 16*half + 8*(lane/32) + e of output channel m = 32j + lane%32.
// Forward reads w[tap][k][m]; data-grad reads w[26-tap][m][k] (taps mirrored, roles swapped), where
// the kernel's input channels are the layer's output channels.  ki / ko = channel counts as the
// kernel sees them (ki in, ko out).
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t *__restrict__ w,
                                                           uint16_t *__restrict__ wpack, int ki, int ko,
                                                           int dgrad, int flat) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int per_pair = NFRAG * 64 * 8;
    const int pairs = (ki / C) * (ko / C);
    if (idx >= per_pair * pairs) return;
    const int pair = idx / per_pair, i = idx % per_pair;
    const int ci = pair / (ko / C), cj = pair % (ko / C);
    const int e = i & 7, lane = (i >> 3) & 63, half = (i >> 9) & 1, tap = i >> 10;
    const int m = C * cj + (lane & 31), k = C * ci + 16 * half + 8 * (lane >> 5) + e;
    // forward: w[tap][cin = k][cout = m] (row length ko); dgrad: w[26-tap][cin = m][cout = k] (row length ki)
    if (flat) {
        // w[3][3][..][..]: its 9 taps are the kernel's taps 9..17 (kd = 1); the other fragments are never loaded
        // and stay unwritten
        const int t9 = tap - 9;
        if (t9 >= 0 && t9 < 9)
            wpack[idx] = dgrad ? w[(static_cast<size_t>(8 - t9) * ko + m) * ki + k]
                               : w[(static_cast<size_t>(t9) * ki + k) * ko + m];
        return;
    }
    wpack[idx] = dgrad ? w[(static_cast<size_t>(26 - tap) * ko + m) * ki + k]
                       : w[(static_cast<size_t>(tap) * ki + k) * ko + m];
}

// two floats -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack2(float a, float b) {
    union { bf16x2 v; uint32_t u; } r;
    r.v = __builtin_convertvector(f32x2{a, b}, bf16x2);
    return r.u;
}

// Where output block cj goes: tensor, its channels per voxel, channel offset.
struct OutDst { uint16_t *base; int cs, co; };
__device__ __forceinline__ OutDst out_dest(const ConvArgs &a, int cj) {
    if (a.out2 && C * cj >= a.out_ca) return OutDst{a.out2, a.out2_cs, C * cj - a.out_ca};
    return OutDst{a.out, a.out_cs, C * cj};
}

// What happens to a finished output value (template parameter RELU of the kernels below).
enum Epilogue { kNone = 0, kRelu = 1,   // max(z, 0): forward with SP_FLAG_RELU
                kMask = 2,              // z where the mask tensor is positive, else 0: the data gradient followed
                                        // by the backward of the ReLU that produced the layer's input
                kMaskBits = 3,          // kMask with the one-bit form of the mask
                kReluBits = 4 };        // kRelu that also writes the one-bit mask of its result
constexpr bool is_relu(int e) { return e == kRelu || e == kReluBits; }

// One-bit ReLU mask.  The masked data gradient needs of the activation only "was it positive"; as a tensor that
// costs a second full read (64 bytes per voxel and 32 channels), as bits 4 bytes.  The bits are kept in the order
// in which the matrix cores hand results to the lanes, so that neither side has to shuffle: per padded voxel and
// block of 32 channels two 16-bit words, word `hi` holding channel 8 q + 4 hi + i in bit 4 q + i (q = 0..3,
// i = 0..3) - exactly the 16 values that lane 32 hi + voxel holds for a row.  Word index:
// (padded voxel index * blocks + block) * 2 + hi.  Only interior voxels are ever written or read.
// A bit is set where the bf16 value is positive: not zero, not negative, not NaN (positive_halves).

// two bf16 in a word -> 0xffff in each half whose value is positive (not zero, not negative, not NaN)
__device__ __forceinline__ uint32_t positive_halves(uint32_t v) {
    const uint32_t lo = v & 0xffffu, hi = v >> 16;
    return ((lo - 1u) < 0x7f80u ? 0x0000ffffu : 0u) | ((hi - 1u) < 0x7f80u ? 0xffff0000u : 0u);
}

// Partial sums and mask values of one store unit, in vector types that can be operands of the
// assembly below.
typedef float pin_t __attribute__((ext_vector_type(4)));
typedef uint32_t mask_t __attribute__((ext_vector_type(2)));

// Side loads: loads that the compiler does not see.  Whenever a register filled by an ordinary global load
// is first used, the compiler drains the vector-memory queue far enough for that load - and, since it
// cannot order the staging loads (which write LDS, or are assembly themselves) against it, in effect the
// whole queue: s_waitcnt vmcnt(0) or nearly so, once per plane step, with three planes of staging loads in
// flight.  Every kernel that reads partial sums or a mask paid a full memory latency per step for it.
// Where registers allow, those values are therefore fetched by assembly at the START of the step BEFORE the
// one that uses them, into a second set of registers.  Vector-memory operations complete in issue order and
// a step issues its staging loads and stores after them, so the wait that ends every step (at most
// (DIST - 1) * LOADS operations outstanding) already covers them: the registers pass through that wait as
// operands (side_fence), nothing reads them earlier, and they hold their data at every block boundary, where
// the compiler is free to copy them.  The step that uses them needs no wait at all.  Marches over ragged
// patches, whose loads are predicated, keep the ordinary loads.
__device__ __forceinline__ void side_load(pin_t &d, const float *p) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(d) : "v"(p) : "memory");
}
__device__ __forceinline__ void side_load(mask_t &d, const uint16_t *p) {
    asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(d) : "v"(p) : "memory");
}
// (a macro: a reference cannot bind to the vector element that receives the word)
#define SP3D_SIDE_LOAD_BITS(d, p) asm volatile("global_load_ushort %0, %1, off" : "=v"(d) : "v"(p) : "memory")
// The wait of a step's end (NV vector-memory operations may stay outstanding; LG: LDS operations must have
// finished as well) with the side registers as operands.
#define SP3D_SIDE8(a) "+v"(a[0][0]), "+v"(a[0][1]), "+v"(a[0][2]), "+v"(a[0][3]), "+v"(a[1][0]), "+v"(a[1][1]), \
                      "+v"(a[1][2]), "+v"(a[1][3])
#define SP3D_SIDE2(a) "+v"(a[0][0].x), "+v"(a[1][0].x)      // the bit form: one word per row, kept in [row][0].x
template <int NV, bool LG, bool PINS, bool MASK, bool BITS>
__device__ __forceinline__ void side_fence(pin_t (&p)[2][4], mask_t (&m)[2][4]) {
    static_assert(!BITS || MASK, "the bit form is a form of the mask");
    if (LG) {
        if (PINS && BITS) asm volatile("s_waitcnt vmcnt(%10) lgkmcnt(0)" : SP3D_SIDE8(p), SP3D_SIDE2(m) : "n"(NV) : "memory");
        else if (PINS && MASK) asm volatile("s_waitcnt vmcnt(%16) lgkmcnt(0)" : SP3D_SIDE8(p), SP3D_SIDE8(m) : "n"(NV) : "memory");
        else if (PINS) asm volatile("s_waitcnt vmcnt(%8) lgkmcnt(0)" : SP3D_SIDE8(p) : "n"(NV) : "memory");
        else if (BITS) asm volatile("s_waitcnt vmcnt(%2) lgkmcnt(0)" : SP3D_SIDE2(m) : "n"(NV) : "memory");
        else if (MASK) asm volatile("s_waitcnt vmcnt(%8) lgkmcnt(0)" : SP3D_SIDE8(m) : "n"(NV) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NV) : "memory");
    } else {
        if (PINS && BITS) asm volatile("s_waitcnt vmcnt(%10)" : SP3D_SIDE8(p), SP3D_SIDE2(m) : "n"(NV) : "memory");
        else if (PINS && MASK) asm volatile("s_waitcnt vmcnt(%16)" : SP3D_SIDE8(p), SP3D_SIDE8(m) : "n"(NV) : "memory");
        else if (PINS) asm volatile("s_waitcnt vmcnt(%8)" : SP3D_SIDE8(p) : "n"(NV) : "memory");
        else if (BITS) asm volatile("s_waitcnt vmcnt(%2)" : SP3D_SIDE2(m) : "n"(NV) : "memory");
        else if (MASK) asm volatile("s_waitcnt vmcnt(%8)" : SP3D_SIDE8(m) : "n"(NV) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NV) : "memory");
    }
}
#undef SP3D_SIDE8
#undef SP3D_SIDE2
// What a kernel variant fetches per store unit besides its operands, and whether it does so by side loads.
// Measured: the mask gains from them (3-D 32 -> 32 at 512^3: 7.45 -> 7.08 ms; 2-D: 8 - 9 %) except in the 3-D
// two-chunk kernel, whose registers are all taken (4.07 -> 4.71 ms with them); the partial sums do not gain
// (their cost was the access pattern, see part_unit), so they stay ordinary loads.
template <int MODE, int RELU, int KD, bool PAIR> struct Side {
    static constexpr bool PINS = MODE == kMiddle || MODE == kLast;
    static constexpr bool MASK = (RELU == kMask || RELU == kMaskBits) && (MODE == kSingle || MODE == kLast);
    static constexpr bool BITS = MASK && RELU == kMaskBits;      // one 16-bit word per row instead of 4 x 8 bytes
    static constexpr bool ASYNC = MASK && !PINS && (KD == 1 || !PAIR || BITS);
};
// Role of a step in the chain of side loads.
enum SideStep { kSideNone = 0,     // no side loads (nothing to fetch, or a ragged patch)
                kSideFetch = 1,    // fetch for the next step, nothing to use yet
                kSideUse = 2 };    // use what the previous step fetched, fetch for the next

// fp32 partial sums between the launches of a layer are kept in FRAGMENT order, not in the layout of the
// output tensor: every launch of the layer has the same decomposition into workgroups and waves, so a wave
// reads back exactly what the same wave of the previous launch wrote, and what a wave moves per store unit
// (64 lanes x 4 channels) is one contiguous kilobyte - lane l at byte 16 l.  (In tensor order the 16 bytes of
// neighbouring lanes lie a whole voxel record apart, 4 KB at 1024 channels, and a wave-wide access touches 64
// cache lines; those accesses, not the arithmetic, bounded the launches of wide layers.)  A wave's region
// holds [plane of the D chunk][row][unit][lane]; part_unit() is the float offset of a unit inside it.
__device__ __forceinline__ size_t part_unit(int d, int h, int q) { return static_cast<size_t>((d * RH + h) * 4 + q) * 256; }

// Offset, in 16-bit words of the one-bit mask, of row h of output plane d from a lane's base: one word per voxel,
// channel block and half, against 16 elements in the tensor.
template <class CtxT>
__device__ __forceinline__ size_t bits_off(const CtxT &c, int d, int h) { return (d * c.oplane + h * c.orow) >> 4; }

// The four bits of a finished store unit, taken from the fp32 values before they are rounded: a value is stored
// as a positive bf16 exactly if it exceeds 2^-134, the midpoint between zero and the smallest bf16 denormal (a tie
// rounds to the even neighbour, zero; fp32 denormals are kept in these kernels' floating-point mode).  NaN compares
// false and +inf true, as the sign test on the stored value has it.  One compare and one select per value, against
// four integer operations on the packed halves.
__device__ __forceinline__ uint32_t positive_nibble(float v0, float v1, float v2, float v3) {
    constexpr float T = 0x1p-134f;
    return (v0 > T ? 1u : 0u) | (v1 > T ? 2u : 0u) | (v2 > T ? 4u : 0u) | (v3 > T ? 8u : 0u);
}
// ... and the reverse: 0xffff in each half of the two words whose bit is set
__device__ __forceinline__ uint2 nibble_halves(uint32_t word, int q) {
    const uint32_t n = word >> (4 * q);
    return make_uint2(((n & 1u) ? 0x0000ffffu : 0u) | ((n & 2u) ? 0xffff0000u : 0u),
                      ((n & 4u) ? 0x0000ffffu : 0u) | ((n & 8u) ? 0xffff0000u : 0u));
}

// kReluBits: write the mask word of row h of plane d that the four store units of the row collected.
template <bool FULL, class CtxT>
__device__ __forceinline__ void store_bits(const CtxT &c, int d, const mask_t (&mk)[RH][4], int h) {
    if (FULL || c.okrow[h]) c.bbase[bits_off(c, d, h)] = static_cast<uint16_t>(mk[h][0].x);
}

// Per-wave state of the march that the side work of a step needs.
template <bool HAS_BIAS>
struct Ctx {
    const uint16_t *tin0;       // first padded input plane of this workgroup's D chunk (at the chunk's channels)
    size_t plane_elems;         // input elements per padded plane of the tile
    int nplanes;                // input planes of the chunk (output planes + 2)
    int plo, phi;               // staged planes are clamped to [plo, phi] (slices side by side: the outer two are not real)
    ptrdiff_t dlo, dhi;         // gathered halos: what to add for staged plane 0 / the last one (else 0)
    int goff[LOADS];            // per-lane source offsets of the staging loads (elements)
    char *lds_stage;            // LDS chunk plane this wave fills (ring slot 0)
    uint16_t *obase;            // output address of (plane 0, first row of the wave, this lane)
    const uint16_t *mbase;      // same position in the mask tensor
    uint16_t *bbase;            // this lane's word of that voxel in the one-bit mask (see relu_bit)
    float *pbase;               // this lane's slot in the wave's region of the fp32 partial-sum buffer
    size_t oplane, orow;        // output elements per padded plane / per padded row
    bool okrow[RH];             // row/column of this lane lies inside the tile interior
    float bv[HAS_BIAS ? 16 : 1];
};

// Staging load j of padded plane `dplane` of the chunk -> ring slot dplane % NBUF.  global_load_lds:
// lane l supplies its own global address and the 16 bytes land at LDS base + 16*l.  Planes past the last
// one needed are clamped (their ring slot is never read), so every step issues exactly LOADS loads.
template <bool HAS_BIAS>
__device__ __forceinline__ void stage(const Ctx<HAS_BIAS> &c, int dplane, int j, int lane) {
    const int dpl = min(max(dplane, c.plo), c.phi);
    const uint16_t *p = c.tin0 + static_cast<ptrdiff_t>(dpl) * static_cast<ptrdiff_t>(c.plane_elems) +
                        (dpl == 0 ? c.dlo : 0) + (dpl == c.nplanes - 1 ? c.dhi : 0);
    char *dst = c.lds_stage + (dplane % NBUF) * PLANE_BYTES + j * 1024;
    if (64 * j + lane < PLANE_VOX)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p + c.goff[j]),
                                         (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
}

// Partial sums of 4 channels of row h of plane d written by the previous input chunk.
template <bool FULL, bool HAS_BIAS>
__device__ __forceinline__ pin_t load_partial(const Ctx<HAS_BIAS> &c, int d, int h, int q) {
    pin_t v = pin_t{0.f, 0.f, 0.f, 0.f};
    if (FULL || c.okrow[h]) v = *reinterpret_cast<const pin_t *>(c.pbase + part_unit(d, h, q));
    return v;
}

// The 4 mask values that belong to one store unit (fetched at the start of the step, like the partial sums).
template <bool FULL, bool BITS, bool HAS_BIAS>
__device__ __forceinline__ mask_t load_mask(const Ctx<HAS_BIAS> &c, int d, int h, int q) {
    mask_t v = mask_t{0u, 0u};
    if (BITS) {         // the row's word, kept in unit 0
        if (q == 0 && (FULL || c.okrow[h])) v.x = c.bbase[bits_off(c, d, h)];
        return v;
    }
    if (FULL || c.okrow[h]) v = *reinterpret_cast<const mask_t *>(c.mbase + d * c.oplane + h * c.orow + 8 * q);
    return v;
}

// Finish 4 channels of row h of a finished plane (channels 8q + 4*(lane/32) .. +3 of this output block):
// add the earlier chunks' partial sums if there are any, then either store the new partial (fp32) or
// apply ReLU, convert and store bf16 (8 bytes).
template <int MODE, int RELU, bool FULL, bool HAS_BIAS>
__device__ __forceinline__ void store_unit(const Ctx<HAS_BIAS> &c, int d, const f32x16 (&s)[RH],
                                           const pin_t (&pin)[RH][4], mask_t (&mk)[RH][4], int h, int q) {
    float v0 = s[h][4 * q], v1 = s[h][4 * q + 1], v2 = s[h][4 * q + 2], v3 = s[h][4 * q + 3];
    if (MODE == kMiddle || MODE == kLast) {
        v0 += pin[h][q].x; v1 += pin[h][q].y; v2 += pin[h][q].z; v3 += pin[h][q].w;
    }
    const size_t at = d * c.oplane + h * c.orow + 8 * q;
    if (MODE == kFirst || MODE == kMiddle) {
        if (FULL || c.okrow[h]) *reinterpret_cast<float4 *>(c.pbase + part_unit(d, h, q)) = make_float4(v0, v1, v2, v3);
        return;
    }
    if (is_relu(RELU)) {
        v0 = v0 < 0.f ? 0.f : v0; v1 = v1 < 0.f ? 0.f : v1;
        v2 = v2 < 0.f ? 0.f : v2; v3 = v3 < 0.f ? 0.f : v3;
    }
    uint2 pk = make_uint2(pack2(v0, v1), pack2(v2, v3));
    if (RELU == kMask) {
        pk.x &= positive_halves(mk[h][q].x);
        pk.y &= positive_halves(mk[h][q].y);
    }
    if (RELU == kMaskBits) {
        const uint2 m = nibble_halves(mk[h][0].x, q);
        pk.x &= m.x;
        pk.y &= m.y;
    }
    if (FULL || c.okrow[h]) *reinterpret_cast<uint2 *>(c.obase + at) = pk;
    if (RELU == kReluBits) {
        // the row's word collects in the (otherwise unused) mask register of unit 0 and leaves with the last unit
        const uint32_t n = positive_nibble(v0, v1, v2, v3) << (4 * q);
        mk[h][0].x = q == 0 ? n : (mk[h][0].x | n);
        if (q == 3) store_bits<FULL>(c, d, mk, h);
    }
}

// All MFMAs of one staged input plane Dp, with the step's side work spread over the six MFMA groups:
// the staging loads of plane Dp+DIST and (EPI) the conversion and stores of output plane Dp-3, which
// received its last contribution in step Dp-1, after which its accumulator slot returns to the bias.
// `lbase` = this lane's read base inside the plane: voxel (first row of the wave, column lane%32),
// chunk lane/32.  Fragments are fetched one (kw, K-half) group of RH+2 rows ahead of the MFMAs that
// consume them.  P = Dp mod 4: output plane Dp-kd lives in slot (P-kd) mod 4, plane Dp-3 in slot (P+1) mod 4.
// FULL: the patch lies completely inside the tile interior, so stores need no mask (no branches in
// the step, which lets the scheduler weave the side work between the MFMAs).
// SIDE (see side_load): kSideNone - the step loads its own partial sums / mask values (pin, mk) the ordinary
// way; otherwise it uses the ones the previous step fetched (kSideUse) and first of all fetches those of the
// plane that the next step finishes, Dp - 2, into the other set (npin, nmk), which the caller passes through
// the wait that ends the step.
template <int P, bool EPI, int MODE, int RELU, bool FULL, int KD, int SIDE, bool HAS_BIAS>
__device__ __forceinline__ void plane_step(const Ctx<HAS_BIAS> &c, int Dp, int lane, const char *lbase,
                                           const bf16x8 (&wf)[NFRAG], f32x16 (&acc)[4][RH],
                                           pin_t (&pin)[RH][4], mask_t (&mk)[RH][4],
                                           pin_t (&npin)[RH][4], mask_t (&nmk)[RH][4]) {
    constexpr int NR = RH + 2;
    constexpr int DONE = (P + 1) & 3;
    using S = Side<MODE, RELU, KD, false>;
    bf16x8 b[2][NR];
    if (SIDE != kSideNone) {
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const size_t at = (Dp - 2) * c.oplane + h * c.orow + 8 * q;
                if (S::PINS) side_load(npin[h][q], c.pbase + part_unit(Dp - 2, h, q));
                if (S::MASK && !S::BITS) side_load(nmk[h][q], c.mbase + at);
                if (S::BITS && q == 0) SP3D_SIDE_LOAD_BITS(nmk[h][0].x, c.bbase + bits_off(c, Dp - 2, h));
            }
    }
    if (SIDE == kSideNone && EPI && S::PINS) {
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int q = 0; q < 4; ++q) pin[h][q] = load_partial<FULL>(c, Dp - 3, h, q);
    }
    if (SIDE == kSideNone && EPI && S::MASK) {
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int q = 0; q < 4; ++q) mk[h][q] = load_mask<FULL, S::BITS>(c, Dp - 3, h, q);
    }
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
                store_unit<MODE, RELU, FULL>(c, Dp - 3, acc[DONE], pin, mk, 0, gi);
                store_unit<MODE, RELU, FULL>(c, Dp - 3, acc[DONE], pin, mk, 1, gi);
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
                    if (KD == 1 && kd != 1) continue;
                    const int slot = (P - kd + 4) & 3;
                    acc[slot][h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        wf[((kd * 3 + kh) * 3 + kw) * 2 + half], b[gi & 1][r], acc[slot][h], 0, 0, 0);
                }
            }
        // weave: after each MFMA let a few of the side-work instructions issue while it executes
#pragma unroll
        for (int i = 0; i < KD * (RH + 1) * 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x006, 3, 0);   // up to three VALU / SALU
            if (i % 6 == 2) __builtin_amdgcn_sched_group_barrier(0x060, 1, 0);   // a vector memory op
        }
    }
}

template <int MODE, bool HAS_BIAS, int RELU, int KD>
__global__ __launch_bounds__(kThreads, 1) void conv_mfma_kernel(ConvArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];   // NBUF planes of PLANE_BYTES
    const Geo &g = a.g;
    // Consecutive hardware workgroup ids rotate over the 8 XCDs; give each XCD a contiguous range of
    // logical ids so that patches sharing halo rows/columns meet in the same L2.
    const int per_xcd = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= a.nblocks) return;
    int t = logical;
    const int cj = t % a.nco; t /= a.nco;          // output block: fastest, so that the workgroups that
                                                    // share an input patch run together
    const int pw_i = t % a.nw; t /= a.nw;
    const int ph_i = t % a.nh; t /= a.nh;
    const int pd_i = t % a.nd; t /= a.nd;
    const int tile = t;
    const int d0 = pd_i * a.dchunk, h0 = ph_i * PH, w0 = pw_i * PW;      // coordinates inside the output box
    const TileBox bx = tile_box(g, tile);
    int dn = min(a.dchunk, bx.bd - d0);                                 // output planes (slices) to produce
    // the patches are laid out for the largest box of the grid; a tile at the volume border has a smaller one
    if (dn <= 0 || h0 >= bx.bh || w0 >= bx.bw) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hi = lane >> 5;

    // weight fragments: 54 x 16 bytes per lane, resident for the whole march
    bf16x8 wf[NFRAG];
#pragma unroll
    for (int f = 0; f < NFRAG; ++f) {
        if (KD == 1 && f / 18 != 1) continue;        // 2-D variant: only the taps with kd = 1 exist
        const uint4 q = a.wpack[(cj * NFRAG + f) * 64 + lane];
        wf[f] = *reinterpret_cast<const bf16x8 *>(&q);
    }

    Ctx<HAS_BIAS> c;
    const int F = KD == 1 ? a.fold : 1;         // slices side by side (see fold_col); dn is a multiple of F
    const size_t plane_real = static_cast<size_t>(g.ph) * g.pw * a.in_cs;
    c.plane_elems = plane_real * F;
    c.tin0 = a.in + (static_cast<size_t>(tile) * g.tile_vox + bx.org) * a.in_cs + d0 * plane_real + a.in_co -
             static_cast<ptrdiff_t>(F - 1) * static_cast<ptrdiff_t>(plane_real);
    dn /= F;                                    // from here on: output steps
    c.nplanes = dn + 2;
    c.plo = F > 1 ? 1 : 0;
    c.phi = F > 1 ? c.nplanes - 2 : c.nplanes - 1;
    // Wave w fills chunk plane w (channels 8w..8w+7 of every voxel); load j covers patch-local voxels
    // 64j..64j+63.  Voxels beyond the box and its one-voxel surround (ragged patches) are clamped to a valid
    // address; they only feed outputs that are never stored.
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int v = 64 * j + lane;
        const FoldCol fc = fold_col(v % LCOLS, F, a.fold_w);
        const int row = min(h0 + v / LCOLS, bx.bh + 1), colv = min(w0 + fc.c, bx.bw + 1);
        c.goff[j] = ((min(fc.s, F - 1) * g.ph + row) * g.pw + colv) * a.in_cs + wave * 8;
    }
    c.dlo = c.dhi = 0;
    if (a.gather) {          // (host: one-voxel margins, no grown box, 3-D)
        const GatherShift gs = gather_shift(g, tile, a.in_cs);
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const int v = 64 * j + lane;
            const int row = min(h0 + v / LCOLS, bx.bh + 1), colv = min(w0 + v % LCOLS, bx.bw + 1);
            c.goff[j] += (row == 0 ? gs.hm : 0) + (row == g.th + 1 ? gs.hp : 0) + (colv == 0 ? gs.wm : 0) +
                         (colv == g.tw + 1 ? gs.wp : 0);
        }
        if (d0 == 0) c.dlo = gs.dm;
        if (d0 + dn == g.td) c.dhi = gs.dp;
    }
    c.lds_stage = lds + wave * CH_STRIDE;
    const OutDst od = out_dest(a, cj);
    const FoldCol oc = fold_col(col, F, a.fold_w);
    c.orow = static_cast<size_t>(g.pw) * od.cs;
    c.oplane = static_cast<size_t>(g.ph) * c.orow * F;
    const size_t ovox = static_cast<size_t>(tile) * g.tile_vox + bx.org +
                        (static_cast<size_t>(d0 + 1 + min(oc.s, F - 1)) * g.ph + h0 + wave * RH + 1) * g.pw + w0 +
                        oc.c + 1;
    const size_t opos = ovox * od.cs + od.co + 4 * hi;
    c.obase = od.base + opos;
    c.mbase = a.mask + opos;
    c.bbase = a.bits + (ovox * a.nco + cj) * 2 + hi;
    // wave `wave` of workgroup `logical`: a region of dchunk planes x RH rows x 4 units x 1 KB
    c.pbase = a.part + (static_cast<size_t>(logical) * kWaves + wave) * a.dchunk * (RH * 4 * 256) + lane * 4;
#pragma unroll
    for (int h = 0; h < RH; ++h) c.okrow[h] = h0 + wave * RH + h < bx.bh && w0 + oc.c < bx.bw && oc.s < F;
    // the bias is folded into the accumulators: a slot starts from the bias instead of zero
    // (without a bias the slots start from the constant zero and no registers are spent on it)
    if (HAS_BIAS) {
#pragma unroll
        for (int i = 0; i < 16; ++i) c.bv[HAS_BIAS ? i : 0] = a.bias[C * cj + 8 * (i >> 2) + 4 * hi + (i & 3)];
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
        using S = Side<MODE, RELU, KD, false>;
        // whole patches fetch their partial sums / mask values one step ahead (see side_load): steps with an even
        // plane index use set A and fetch into set B, odd ones the other way round
        constexpr bool ASYNC = FULL && S::ASYNC;
        constexpr int FETCH = ASYNC ? kSideFetch : kSideNone, USE = ASYNC ? kSideUse : kSideNone;
        pin_t pinA[RH][4], pinB[RH][4];
        mask_t mkA[RH][4], mkB[RH][4];
        // (a step with stores issues LOADS + 8 >= (DIST - 1) * LOADS operations after its side loads; the
        // fetch-only step issues just its LOADS staging loads after them and waits accordingly)
#define SP3D_STEP_END_SIDE(NV, NP, NM)                                                   \
    do {                                                                                 \
        side_fence<NV, false, ASYNC && S::PINS, ASYNC && S::MASK, ASYNC && S::BITS>(NP, NM); \
        __builtin_amdgcn_s_barrier();                                                    \
    } while (0)
        static_assert(LOADS + 8 >= (DIST - 1) * LOADS, "side loads must be older than what the step-end wait lets stay in flight");
        // the first three steps have no finished plane to store (nplanes >= 3 always); the third one fetches
        // what the first store needs
        plane_step<0, false, MODE, RELU, FULL, KD, kSideNone>(c, 0, lane, lbase, wf, acc, pinA, mkA, pinB, mkB);
        SP3D_STEP_END();
        plane_step<1, false, MODE, RELU, FULL, KD, kSideNone>(c, 1, lane, lbase + PLANE_BYTES, wf, acc, pinA, mkA,
                                                              pinB, mkB);
        SP3D_STEP_END();
        plane_step<2, false, MODE, RELU, FULL, KD, FETCH>(c, 2, lane, lbase + 2 * PLANE_BYTES, wf, acc, pinA, mkA,
                                                          pinB, mkB);
        SP3D_STEP_END_SIDE(ASYNC ? LOADS : (DIST - 1) * LOADS, pinB, mkB);
        // steps 3, 4, 5, 6, 7, ...: planes mod 4 = 3, 0, 1, 2, 3, ...
#define SP3D_MAIN_STEP(OFF, PHASE, CP, CM, NP, NM)                                                   \
    if (D + (OFF) < nplanes) {                                                                       \
        plane_step<PHASE, true, MODE, RELU, FULL, KD, USE>(c, D + (OFF), lane, lbase + (PHASE) * PLANE_BYTES, wf, \
                                                           acc, CP, CM, NP, NM);                     \
        SP3D_STEP_END_SIDE((DIST - 1) * LOADS, NP, NM);                                              \
    }
        for (int D = 3; D < nplanes; D += 4) {
            SP3D_MAIN_STEP(0, 3, pinB, mkB, pinA, mkA)
            SP3D_MAIN_STEP(1, 0, pinA, mkA, pinB, mkB)
            SP3D_MAIN_STEP(2, 1, pinB, mkB, pinA, mkA)
            SP3D_MAIN_STEP(3, 2, pinA, mkA, pinB, mkB)
        }
#undef SP3D_MAIN_STEP
#undef SP3D_STEP_END_SIDE
        // the last output plane (dn-1) finished in the last step; it sits in slot (dn-1) mod 4, and with side
        // loads the last step (plane index dn + 1, of the parity of dn - 1) fetched its values: into set B if
        // that index is even
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (!ASYNC && S::PINS) {
#pragma unroll
            for (int h = 0; h < RH; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q) pinA[h][q] = pinB[h][q] = load_partial<FULL>(c, dn - 1, h, q);
        }
        if (!ASYNC && S::MASK) {
#pragma unroll
            for (int h = 0; h < RH; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q) mkA[h][q] = mkB[h][q] = load_mask<FULL, S::BITS>(c, dn - 1, h, q);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
            if (s == ((dn - 1) & 3)) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    store_unit<MODE, RELU, FULL>(c, dn - 1, acc[s], (s & 1) ? pinA : pinB, (s & 1) ? mkA : mkB, 0, q);
                    store_unit<MODE, RELU, FULL>(c, dn - 1, acc[s], (s & 1) ? pinA : pinB, (s & 1) ? mkA : mkB, 1, q);
                }
            }
    };
    if (h0 + PH <= bx.bh && w0 + PW <= bx.bw) march(std::true_type{});
    else march(std::false_type{});
#undef SP3D_STEP_END
}

// =============================================================================================
// Two input chunks per launch (layers with Cin a multiple of 64).  With one chunk per launch every extra
// chunk costs a round trip of the fp32 partial sums through HBM (8 bytes per output value), which makes
// wide layers bandwidth-bound.  Here a workgroup contracts 64 input channels at once and adds the two
// halves on chip: the patch is 4 rows x 32 columns, waves 0, 1 take input chunk 0 and waves 2, 3 chunk 1
// of the pair, each for one row group of 2 rows, with the same register-resident weights, D march and
// fragment reuse as above.  When an output plane is complete, the chunk-1 wave writes its 2 x 16
// accumulators to a small LDS buffer (during the next step, between its MFMAs); one step later, after the
// step barrier, the chunk-0 wave of the same rows adds them to its own, converts and stores.  A plane
// therefore lives in an accumulator slot for five steps (three contributing, one being handed over, one
// being stored), hence five slots.  Layers with more than one pair still go through fp32 partial sums, but
// half as often.
namespace wide {

constexpr int NRG = 2;                      // row groups
constexpr int PH = RH * NRG;                // 4 patch rows
constexpr int LROWS = PH + 2;               // 6
constexpr int PLANE_VOX = LROWS * LCOLS;    // 204 voxels of one chunk's plane
constexpr int CP_LOADS = (PLANE_VOX + 63) / 64;      // 4 wave loads per 16-byte chunk plane
constexpr int LOADS = 2 * CP_LOADS;         // a wave fills two of the four chunk planes of its input chunk
constexpr int NSLOT = 5;
constexpr int CH_STRIDE = (PLANE_VOX + 2) * 16;      // 3296
constexpr int CHUNK_BYTES = 4 * CH_STRIDE;           // 13184: one input chunk's plane
constexpr int PLANE_BYTES = 2 * CHUNK_BYTES;         // both chunks of the pair
constexpr int RING_BYTES = NBUF * PLANE_BYTES;       // 105472
constexpr int RED_BYTES = NRG * RH * 4 * 64 * 16;    // 16384: one plane's hand-over (float4 per lane and unit)
// Weight fragments in LDS (3-D kernel).  A wave needs 54 fragments = 216 registers beside 160 accumulators, and
// the register allocation of these kernels was over its 512 by 30 - 80 registers: the compiler spilled weight
// fragments to scratch and reloaded them at their use, 1 - 7 times per plane step, and since it cannot tell its own
// scratch load from the staging loads in flight it followed every reload with a wait for ALL outstanding memory
// operations - the prefetch of three planes drained several times per step.  The twelve fragments of the taps with
// kh = 2 and kd = 1, 2 (the ones a group of MFMAs uses last) therefore live in LDS, once per input chunk of the
// pair (both waves of a chunk use the same ones), and are read at the start of the group that uses them: a read
// the LDS counter tracks, no memory wait.
constexpr int WL_FRAGS = 12;
constexpr int WL_BYTES = 2 * WL_FRAGS * 1024;          // 24576: both input chunks of the pair
constexpr int WL_BASE = RING_BYTES + 2 * RED_BYTES;
constexpr int LDS_BYTES = WL_BASE + WL_BYTES;          // 162816
static_assert(LDS_BYTES <= 160 * 1024, "LDS of one CU");
__host__ __device__ constexpr bool wl_in_lds(int KD, int f) {      // fragment f = (tap, half)
    return KD == 3 && ((f / 2) / 3) % 3 == 2 && (f / 2) / 9 >= 1;
}
__host__ __device__ constexpr int wl_index(int kd, int kw, int half) { return ((kd - 1) * 3 + kw) * 2 + half; }

// direct-to-LDS load as in wgrad_mfma.hip: written as assembly so that the compiler neither tracks it nor
// drains it before unrelated LDS accesses; the kernel counts the loads itself (s_waitcnt vmcnt)
__device__ __forceinline__ void dma16(const uint16_t *src, const char *dst) {
    const uint32_t l = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (const __attribute__((address_space(3))) char *)dst));
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(l) : "memory");
}

template <bool HAS_BIAS>
struct Ctx {
    const uint16_t *tin0;       // first padded input plane of the D chunk, at this wave's input chunk
    size_t plane_elems;
    int nplanes;
    int plo, phi;               // staged planes are clamped to [plo, phi]
    ptrdiff_t dlo, dhi;         // gathered halos: what to add for staged plane 0 / the last one (else 0)
    int goff[LOADS];            // source offsets of the staging loads (elements)
    bool tail_lane;             // lane has a voxel in the last (partial) load of a chunk plane
    char *lds_stage;            // first chunk plane this wave fills, ring slot 0
    char *red;                  // hand-over buffer of this wave's row group (buffer 0), lane part included
    const char *wl;             // this chunk's LDS-resident weight fragments, lane part included
    uint16_t *obase;
    const uint16_t *mbase;
    uint16_t *bbase;
    float *pbase;
    size_t oplane, orow;
    bool okrow[RH];
    float bv[HAS_BIAS ? 16 : 1];
};

// staging load j (0..7) of plane `dplane`: chunk plane j / 4 of this wave's two, voxels 64 (j % 4) ..
template <bool HAS_BIAS>
__device__ __forceinline__ void stage(const Ctx<HAS_BIAS> &c, int dplane, int j) {
    const int dpl = min(max(dplane, c.plo), c.phi);
    const uint16_t *p = c.tin0 + static_cast<ptrdiff_t>(dpl) * static_cast<ptrdiff_t>(c.plane_elems) +
                        (dpl == 0 ? c.dlo : 0) + (dpl == c.nplanes - 1 ? c.dhi : 0);
    const char *dst = c.lds_stage + (dplane % NBUF) * PLANE_BYTES + (j / CP_LOADS) * CH_STRIDE + (j % CP_LOADS) * 1024;
    // only the last load of a chunk plane is partial (204 = 3 x 64 + 12 voxels); j is a compile-time constant
    // at every call site, so the other loads carry no predicate
    if (j % CP_LOADS != CP_LOADS - 1 || c.tail_lane) dma16(p + c.goff[j], dst);
}

template <bool FULL, bool HAS_BIAS>
__device__ __forceinline__ pin_t load_partial(const Ctx<HAS_BIAS> &c, int d, int h, int q) {
    pin_t v = pin_t{0.f, 0.f, 0.f, 0.f};
    if (FULL || c.okrow[h]) v = *reinterpret_cast<const pin_t *>(c.pbase + part_unit(d, h, q));
    return v;
}

template <bool FULL, bool BITS, bool HAS_BIAS>
__device__ __forceinline__ mask_t load_mask(const Ctx<HAS_BIAS> &c, int d, int h, int q) {
    mask_t v = mask_t{0u, 0u};
    if (BITS) {         // the row's word, kept in unit 0
        if (q == 0 && (FULL || c.okrow[h])) v.x = c.bbase[bits_off(c, d, h)];
        return v;
    }
    if (FULL || c.okrow[h]) v = *reinterpret_cast<const mask_t *>(c.mbase + d * c.oplane + h * c.orow + 8 * q);
    return v;
}

// chunk-0 wave: finish 4 channels of row h of plane d: own sum + the partner's (from LDS) + earlier pairs'
// partial sums (pin, fetched at the start of the step), then store the new partial (fp32) or ReLU /
// convert / store bf16
template <int MODE, int RELU, bool FULL, bool HAS_BIAS>
__device__ __forceinline__ void finish_unit(const Ctx<HAS_BIAS> &c, int d, const f32x16 (&s)[RH], const char *red,
                                            const pin_t (&pin)[RH][4], mask_t (&mk)[RH][4], int h, int q) {
    const float4 o = *reinterpret_cast<const float4 *>(red + (h * 4 + q) * 1024);
    float v0 = s[h][4 * q] + o.x, v1 = s[h][4 * q + 1] + o.y, v2 = s[h][4 * q + 2] + o.z, v3 = s[h][4 * q + 3] + o.w;
    if (MODE == kMiddle || MODE == kLast) {
        v0 += pin[h][q].x; v1 += pin[h][q].y; v2 += pin[h][q].z; v3 += pin[h][q].w;
    }
    const size_t at = d * c.oplane + h * c.orow + 8 * q;
    if (MODE == kFirst || MODE == kMiddle) {
        if (FULL || c.okrow[h]) *reinterpret_cast<float4 *>(c.pbase + part_unit(d, h, q)) = make_float4(v0, v1, v2, v3);
        return;
    }
    if (is_relu(RELU)) {
        v0 = v0 < 0.f ? 0.f : v0; v1 = v1 < 0.f ? 0.f : v1;
        v2 = v2 < 0.f ? 0.f : v2; v3 = v3 < 0.f ? 0.f : v3;
    }
    uint2 pk = make_uint2(pack2(v0, v1), pack2(v2, v3));
    if (RELU == kMask) {
        pk.x &= positive_halves(mk[h][q].x);
        pk.y &= positive_halves(mk[h][q].y);
    }
    if (RELU == kMaskBits) {
        const uint2 m = nibble_halves(mk[h][0].x, q);
        pk.x &= m.x;
        pk.y &= m.y;
    }
    if (FULL || c.okrow[h]) *reinterpret_cast<uint2 *>(c.obase + at) = pk;
    if (RELU == kReluBits) {
        // the row's word collects in the (otherwise unused) mask register of unit 0 and leaves with the last unit
        const uint32_t n = positive_nibble(v0, v1, v2, v3) << (4 * q);
        mk[h][0].x = q == 0 ? n : (mk[h][0].x | n);
        if (q == 3) store_bits<FULL>(c, d, mk, h);
    }
}

// chunk-1 wave: hand 4 channels of row h of a complete plane over to the chunk-0 wave
__device__ __forceinline__ void give_unit(const f32x16 (&s)[RH], char *red, int h, int q) {
    *reinterpret_cast<float4 *>(red + (h * 4 + q) * 1024) =
        make_float4(s[h][4 * q], s[h][4 * q + 1], s[h][4 * q + 2], s[h][4 * q + 3]);
}

// One staged input plane Dp.  P = Dp mod 5: output plane Dp - kd accumulates in slot (P - kd) mod 5.
// ROLE 1 (chunk 1): GIVE = plane Dp - 3 (slot (P + 2) mod 5) goes to the hand-over buffer Dp & 1 and its
// slot is cleared.  ROLE 0 (chunk 0): FIN = plane Dp - 4 (slot (P + 1) mod 5) is finished from the buffer
// written in the previous step, (Dp - 1) & 1, and its slot returns to the bias.
// SIDE (chunk-0 wave; see side_load): kSideNone - the step loads its own partial sums / mask values (pin, mk)
// the ordinary way; otherwise it uses the ones the previous step fetched (kSideUse) and first of all fetches
// those of the plane that the next step finishes, Dp - 3, into the other set (npin, nmk), which the caller
// passes through the wait that ends the step.
template <int P, int ROLE, bool GIVE, bool FIN, int MODE, int RELU, bool FULL, int KD, int SIDE, bool HAS_BIAS>
__device__ __forceinline__ void plane_step(const Ctx<HAS_BIAS> &c, int Dp, const char *lbase,
                                           const bf16x8 (&wf)[NFRAG], f32x16 (&acc)[NSLOT][RH],
                                           pin_t (&pin)[RH][4], mask_t (&mk)[RH][4],
                                           pin_t (&npin)[RH][4], mask_t (&nmk)[RH][4]) {
    constexpr int NR = RH + 2;
    constexpr int SSLOT = ROLE == 1 ? (P + 2) % NSLOT : (P + 1) % NSLOT;     // slot of the side work
    constexpr int NEXT = (P + 1) % NSLOT;      // slot of output plane Dp + 1: must be clean when this step ends
    constexpr bool ACTIVE = ROLE == 1 ? GIVE : FIN;
    using S = Side<MODE, RELU, KD, true>;
    bf16x8 b[2][NR];
    char *red_w = c.red + (Dp & 1) * RED_BYTES;
    const char *red_r = c.red + ((Dp - 1) & 1) * RED_BYTES;
    if (ROLE == 0 && SIDE != kSideNone) {
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const size_t at = (Dp - 3) * c.oplane + h * c.orow + 8 * q;
                if (S::PINS) side_load(npin[h][q], c.pbase + part_unit(Dp - 3, h, q));
                if (S::MASK && !S::BITS) side_load(nmk[h][q], c.mbase + at);
                if (S::BITS && q == 0) SP3D_SIDE_LOAD_BITS(nmk[h][0].x, c.bbase + bits_off(c, Dp - 3, h));
            }
    }
    if (SIDE == kSideNone && ROLE == 0 && FIN && S::PINS) {
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int q = 0; q < 4; ++q) pin[h][q] = load_partial<FULL>(c, Dp - 4, h, q);
    }
    if (SIDE == kSideNone && ROLE == 0 && FIN && S::MASK) {
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int q = 0; q < 4; ++q) mk[h][q] = load_mask<FULL, S::BITS>(c, Dp - 4, h, q);
    }
#pragma unroll
    for (int r = 0; r < NR; ++r) b[0][r] = *reinterpret_cast<const bf16x8 *>(lbase + (r * LCOLS) * 16);
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
        // the two weight fragments of this group that live in LDS (see WL_FRAGS); the MFMAs that use them are
        // the last of the group
        bf16x8 wl2[2];
        if (KD == 3) {
            wl2[0] = *reinterpret_cast<const bf16x8 *>(c.wl + wl_index(1, kw, half) * 1024);
            wl2[1] = *reinterpret_cast<const bf16x8 *>(c.wl + wl_index(2, kw, half) * 1024);
        }
        __builtin_amdgcn_sched_barrier(0);
        // eight staging loads over six groups
        stage(c, Dp + DIST, gi);
        if (gi < 2) stage(c, Dp + DIST, NG + gi);
        if (gi < 4) {
            if (ACTIVE) {
                if (ROLE == 1) {
                    give_unit(acc[SSLOT], red_w, 0, gi);
                    give_unit(acc[SSLOT], red_w, 1, gi);
                } else {
                    finish_unit<MODE, RELU, FULL>(c, Dp - 4, acc[SSLOT], red_r, pin, mk, 0, gi);
                    finish_unit<MODE, RELU, FULL>(c, Dp - 4, acc[SSLOT], red_r, pin, mk, 1, gi);
                }
            }
        } else {
            // the slot of the next output plane starts from the bias (chunk 0) or zero (chunk 1); in the first
            // steps it holds sums for planes that do not exist.  A handed-over slot is cleared as well.
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                acc[NEXT][gi - 4][i] = (ROLE == 0 && HAS_BIAS) ? c.bv[HAS_BIAS ? i : 0] : 0.f;
                if (ROLE == 1 && GIVE) acc[SSLOT][gi - 4][i] = 0.f;
            }
        }
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const int h = r - kh;
                if (h < 0 || h >= RH) continue;
#pragma unroll
                for (int kd = 0; kd < 3; ++kd) {
                    if (KD == 1 && kd != 1) continue;
                    const int slot = (P - kd + NSLOT) % NSLOT;
                    const int f = ((kd * 3 + kh) * 3 + kw) * 2 + half;
                    acc[slot][h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        wl_in_lds(KD, f) ? wl2[kd - 1] : wf[f], b[gi & 1][r], acc[slot][h], 0, 0, 0);
                }
            }
#pragma unroll
        for (int i = 0; i < KD * (RH + 1) * 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x006, 3, 0);   // up to three VALU / SALU
            if (i % 6 == 2) __builtin_amdgcn_sched_group_barrier(0x060, 1, 0);   // a vector memory op
        }
    }
}

// The two steps after the last input plane: only the side work is left.  Dp = nplanes: chunk 1 hands over
// the last output plane (Dp - 3 = dn - 1), chunk 0 finishes plane Dp - 4; Dp = nplanes + 1: chunk 0 finishes
// the last plane.  Same slot arithmetic as plane_step, so every accumulator index stays a constant.
template <int P, int ROLE, bool GIVE, bool FIN, int MODE, int RELU, bool FULL, int KD, int SIDE, bool HAS_BIAS>
__device__ __forceinline__ void drain_step(const Ctx<HAS_BIAS> &c, int Dp, f32x16 (&acc)[NSLOT][RH],
                                           pin_t (&pin)[RH][4], mask_t (&mk)[RH][4],
                                           pin_t (&npin)[RH][4], mask_t (&nmk)[RH][4]) {
    constexpr int SSLOT = ROLE == 1 ? (P + 2) % NSLOT : (P + 1) % NSLOT;
    using S = Side<MODE, RELU, KD, true>;
    // side loads: the first drain step, and a step 3 that is one already (a march of three planes), fetch for
    // the step after them like a plane step
    if (ROLE == 0 && SIDE != kSideNone && Dp <= c.nplanes) {
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const size_t at = (Dp - 3) * c.oplane + h * c.orow + 8 * q;
                if (S::PINS) side_load(npin[h][q], c.pbase + part_unit(Dp - 3, h, q));
                if (S::MASK && !S::BITS) side_load(nmk[h][q], c.mbase + at);
                if (S::BITS && q == 0) SP3D_SIDE_LOAD_BITS(nmk[h][0].x, c.bbase + bits_off(c, Dp - 3, h));
            }
    }
    if (ROLE == 1) {
        if (GIVE && Dp == c.nplanes) {
            char *red_w = c.red + (Dp & 1) * RED_BYTES;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                give_unit(acc[SSLOT], red_w, 0, q);
                give_unit(acc[SSLOT], red_w, 1, q);
            }
        }
    } else if (FIN) {
        const char *red_r = c.red + ((Dp - 1) & 1) * RED_BYTES;
        if (SIDE == kSideNone && S::PINS) {
#pragma unroll
            for (int h = 0; h < RH; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q) pin[h][q] = load_partial<FULL>(c, Dp - 4, h, q);
        }
        if (SIDE == kSideNone && S::MASK) {
#pragma unroll
            for (int h = 0; h < RH; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q) mk[h][q] = load_mask<FULL, S::BITS>(c, Dp - 4, h, q);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            finish_unit<MODE, RELU, FULL>(c, Dp - 4, acc[SSLOT], red_r, pin, mk, 0, q);
            finish_unit<MODE, RELU, FULL>(c, Dp - 4, acc[SSLOT], red_r, pin, mk, 1, q);
        }
    }
}

template <int ROLE, int MODE, bool HAS_BIAS, int RELU, int KD>
__device__ __forceinline__ void run(const ConvArgs &a, char *lds, int logical, int tile, const TileBox &bx, int d0,
                                    int h0, int w0, int dn, int cj, int rg) {
    const Geo &g = a.g;
    const int lane = threadIdx.x & 63;
    const int col = lane & 31, hi = lane >> 5;

    bf16x8 wf[NFRAG];
    {
        const uint4 *wp = a.wpack + static_cast<size_t>(ROLE) * a.nco * NFRAG * 64;     // chunk ROLE of the pair
#pragma unroll
        for (int f = 0; f < NFRAG; ++f) {
            if (KD == 1 && f / 18 != 1) continue;
            const uint4 q = wp[(cj * NFRAG + f) * 64 + lane];
            if (wl_in_lds(KD, f)) {      // both waves of a chunk write the same bytes
                const int tap = f / 2;
                *reinterpret_cast<uint4 *>(lds + WL_BASE + (ROLE * WL_FRAGS + wl_index(tap / 9, tap % 3, f & 1)) * 1024 +
                                           lane * 16) = q;
            } else {
                wf[f] = *reinterpret_cast<const bf16x8 *>(&q);
            }
        }
    }

    Ctx<HAS_BIAS> c;
    const uint16_t *src = ROLE ? a.in2 : a.in;
    const int src_cs = ROLE ? a.in2_cs : a.in_cs, src_co = ROLE ? a.in2_co : a.in_co;
    const int F = KD == 1 ? a.fold : 1;         // slices side by side (see fold_col); dn counts output steps
    const size_t plane_real = static_cast<size_t>(g.ph) * g.pw * src_cs;
    c.plane_elems = plane_real * F;
    c.tin0 = src + (static_cast<size_t>(tile) * g.tile_vox + bx.org) * src_cs + d0 * plane_real + src_co -
             static_cast<ptrdiff_t>(F - 1) * static_cast<ptrdiff_t>(plane_real);
    c.nplanes = dn + 2;
    c.plo = F > 1 ? 1 : 0;
    c.phi = F > 1 ? c.nplanes - 2 : c.nplanes - 1;
    // this wave fills chunk planes 2 rg and 2 rg + 1 (channels 16 rg .. 16 rg + 15) of its input chunk
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int v = 64 * (j % CP_LOADS) + lane;
        const FoldCol fc = fold_col(v % LCOLS, F, a.fold_w);
        const int row = min(h0 + v / LCOLS, bx.bh + 1), colv = min(w0 + fc.c, bx.bw + 1);
        c.goff[j] = ((min(fc.s, F - 1) * g.ph + row) * g.pw + colv) * src_cs + (2 * rg + j / CP_LOADS) * 8;   // always addressable
    }
    c.dlo = c.dhi = 0;
    if (a.gather) {          // see GatherShift
        const GatherShift gs = gather_shift(g, tile, src_cs);
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const int v = 64 * (j % CP_LOADS) + lane;
            const int row = min(h0 + v / LCOLS, bx.bh + 1), colv = min(w0 + v % LCOLS, bx.bw + 1);
            c.goff[j] += (row == 0 ? gs.hm : 0) + (row == g.th + 1 ? gs.hp : 0) + (colv == 0 ? gs.wm : 0) +
                         (colv == g.tw + 1 ? gs.wp : 0);
        }
        if (d0 == 0) c.dlo = gs.dm;
        if (d0 + dn == g.td) c.dhi = gs.dp;
    }
    c.tail_lane = 64 * (CP_LOADS - 1) + lane < PLANE_VOX;
    c.lds_stage = lds + ROLE * CHUNK_BYTES + 2 * rg * CH_STRIDE;
    c.red = lds + RING_BYTES + rg * (RH * 4 * 1024) + lane * 16;
    c.wl = lds + WL_BASE + ROLE * WL_FRAGS * 1024 + lane * 16;
    const OutDst od = out_dest(a, cj);
    const FoldCol oc = fold_col(col, F, a.fold_w);
    c.orow = static_cast<size_t>(g.pw) * od.cs;
    c.oplane = static_cast<size_t>(g.ph) * c.orow * F;
    const size_t ovox = static_cast<size_t>(tile) * g.tile_vox + bx.org +
                        (static_cast<size_t>(d0 + 1 + min(oc.s, F - 1)) * g.ph + h0 + rg * RH + 1) * g.pw + w0 +
                        oc.c + 1;
    const size_t opos = ovox * od.cs + od.co + 4 * hi;
    c.obase = od.base + opos;
    c.mbase = a.mask + opos;
    c.bbase = a.bits + (ovox * a.nco + cj) * 2 + hi;
    // the chunk-0 wave of row group rg of workgroup `logical`: dchunk planes x RH rows x 4 units x 1 KB
    c.pbase = a.part + (static_cast<size_t>(logical) * NRG + rg) * a.dchunk * (RH * 4 * 256) + lane * 4;
#pragma unroll
    for (int h = 0; h < RH; ++h) c.okrow[h] = h0 + rg * RH + h < bx.bh && w0 + oc.c < bx.bw && oc.s < F;
    if (HAS_BIAS) {
#pragma unroll
        for (int i = 0; i < 16; ++i) c.bv[HAS_BIAS ? i : 0] = a.bias[C * cj + 8 * (i >> 2) + 4 * hi + (i & 3)];
    }
    // the bias is folded into the chunk-0 accumulators; chunk-1 accumulators start from zero
    f32x16 acc[NSLOT][RH];
#pragma unroll
    for (int s = 0; s < NSLOT; ++s)
#pragma unroll
        for (int h = 0; h < RH; ++h)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[s][h][i] = (ROLE == 0 && HAS_BIAS) ? c.bv[HAS_BIAS ? i : 0] : 0.f;

    const char *lbase = lds + ROLE * CHUNK_BYTES + hi * CH_STRIDE + (rg * RH * LCOLS + col) * 16;
    const int nplanes = c.nplanes;

#pragma unroll
    for (int i = 0; i < DIST; ++i)
#pragma unroll
        for (int j = 0; j < LOADS; ++j) stage(c, i, j);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");      // staged planes and the parked weight fragments
    __builtin_amdgcn_s_barrier();

    // End of a step: plane Dp + 1 has landed when at most the loads of planes Dp + 2, Dp + 3 are in flight
    // (loads complete in order; stores share the counter and only make the wait stricter), and this wave's
    // hand-over writes have reached LDS.
#define SP3D_STEP_END()                                                                        \
    do {                                                                                       \
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((DIST - 1) * LOADS) : "memory");   \
        __builtin_amdgcn_s_barrier();                                                          \
    } while (0)

    auto march = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        using S = Side<MODE, RELU, KD, true>;
        // whole patches: the chunk-0 wave fetches its partial sums / mask values one step ahead (see side_load),
        // alternating between two sets of registers
        constexpr bool ASYNC = FULL && ROLE == 0 && S::ASYNC;
        constexpr int FETCH = ASYNC ? kSideFetch : kSideNone, USE = ASYNC ? kSideUse : kSideNone;
        pin_t pinA[RH][4], pinB[RH][4];
        mask_t mkA[RH][4], mkB[RH][4];
        // A step that finishes a plane issues LOADS + 8 operations after its side loads, which the wait at its
        // end lets stay in flight; a fetch-only step issues just its staging loads after them and waits
        // accordingly; a drain step issues no staging loads and waits for everything.
        static_assert(LOADS + 8 >= (DIST - 1) * LOADS, "side loads must be older than what the step-end wait lets stay in flight");
#define SP3D_STEP_END_SIDE(NV, NP, NM)                                              \
    do {                                                                            \
        side_fence<NV, true, ASYNC && S::PINS, ASYNC && S::MASK, ASYNC && S::BITS>(NP, NM); \
        __builtin_amdgcn_s_barrier();                                               \
    } while (0)
        plane_step<0, ROLE, false, false, MODE, RELU, FULL, KD, kSideNone>(c, 0, lbase, wf, acc, pinA, mkA, pinB, mkB);
        SP3D_STEP_END();
        plane_step<1, ROLE, false, false, MODE, RELU, FULL, KD, kSideNone>(c, 1, lbase + PLANE_BYTES, wf, acc, pinA, mkA,
                                                                          pinB, mkB);
        SP3D_STEP_END();
        plane_step<2, ROLE, false, false, MODE, RELU, FULL, KD, kSideNone>(c, 2, lbase + 2 * PLANE_BYTES, wf, acc, pinA,
                                                                          mkA, pinB, mkB);
        SP3D_STEP_END();
        // Steps 3, 4, ... with slot phase Dp mod 5 as a compile-time constant (the ring slot Dp mod 4 is a
        // run-time offset: a period of 20 steps would be needed to make both constants).  The march runs two
        // steps past the last input plane; those only hand over / finish what is left.  Step 3 is the first
        // to hand a plane over (and fetches the side values of step 4), step 4 the first to finish one.
#define SP3D_STEP(DP, PHASE, GIVE_EN, FIN_EN, SIDE_EN, CP, CM, NP, NM)                                     \
    if ((DP) < nplanes) {                                                                                  \
        plane_step<PHASE, ROLE, GIVE_EN, FIN_EN, MODE, RELU, FULL, KD, SIDE_EN>(                           \
            c, (DP), lbase + ((DP) % NBUF) * PLANE_BYTES, wf, acc, CP, CM, NP, NM);                        \
        SP3D_STEP_END_SIDE(((SIDE_EN) == kSideFetch ? LOADS : (DIST - 1) * LOADS), NP, NM);                \
    } else if ((DP) < nplanes + 2) {                                                                       \
        drain_step<PHASE, ROLE, GIVE_EN, FIN_EN, MODE, RELU, FULL, KD, SIDE_EN>(c, (DP), acc, CP, CM, NP, NM); \
        SP3D_STEP_END_SIDE(((SIDE_EN) == kSideNone ? (DIST - 1) * LOADS : 0), NP, NM);                     \
    }
        SP3D_STEP(3, 3, true, false, FETCH, pinA, mkA, pinB, mkB)
        SP3D_STEP(4, 4, true, true, USE, pinB, mkB, pinA, mkA)
        for (int D = 5; D < nplanes + 2; D += NSLOT) {
            SP3D_STEP(D, 0, true, true, USE, pinA, mkA, pinB, mkB)
            SP3D_STEP(D + 1, 1, true, true, USE, pinB, mkB, pinA, mkA)
            SP3D_STEP(D + 2, 2, true, true, USE, pinA, mkA, pinB, mkB)
            SP3D_STEP(D + 3, 3, true, true, USE, pinB, mkB, pinA, mkA)
            SP3D_STEP(D + 4, 4, true, true, USE, pinA, mkA, pinB, mkB)
            // five steps per round: the sets have changed roles
            if (ASYNC) {
#pragma unroll
                for (int h = 0; h < RH; ++h)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const pin_t tp = pinA[h][q]; pinA[h][q] = pinB[h][q]; pinB[h][q] = tp;
                        const mask_t tm = mkA[h][q]; mkA[h][q] = mkB[h][q]; mkB[h][q] = tm;
                    }
            }
        }
#undef SP3D_STEP
#undef SP3D_STEP_END_SIDE
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // clamped staging loads of the last steps
    };
    if (h0 + PH <= bx.bh && w0 + PW <= bx.bw) march(std::true_type{});
    else march(std::false_type{});
#undef SP3D_STEP_END
}

template <int MODE, bool HAS_BIAS, int RELU, int KD>
__global__ __launch_bounds__(kThreads, 1) void conv_mfma_pair_kernel(ConvArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const Geo &g = a.g;
    const int per_xcd = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= a.nblocks) return;
    int t = logical;
    const int cj = t % a.nco; t /= a.nco;
    const int pw_i = t % a.nw; t /= a.nw;
    const int ph_i = t % a.nh; t /= a.nh;
    const int pd_i = t % a.nd; t /= a.nd;
    const int tile = t;
    const int d0 = pd_i * a.dchunk, h0 = ph_i * PH, w0 = pw_i * PW;
    const TileBox bx = tile_box(g, tile);
    const int dn = min(a.dchunk, bx.bd - d0);
    if (dn <= 0 || h0 >= bx.bh || w0 >= bx.bw) return;     // patch of the largest box that this tile's box lacks
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // two copies of the march, one per role, so that each is straight-line code for the scheduler
    const int dsteps = KD == 1 ? dn / a.fold : dn;       // slices side by side: a step produces `fold` of them
    if (wave < 2) run<0, MODE, HAS_BIAS, RELU, KD>(a, lds, logical, tile, bx, d0, h0, w0, dsteps, cj, wave & 1);
    else run<1, MODE, HAS_BIAS, RELU, KD>(a, lds, logical, tile, bx, d0, h0, w0, dsteps, cj, wave & 1);
}

}  // namespace wide

}  // namespace

bool conv_mfma_supported(const Geo &g, int ki, int ko, sp_dtype_t dt) {
    return dt == SP_BF16 && ki % C == 0 && ko % C == 0 && ki <= 1024 && ko <= 1024 &&
           1LL * g.ph * g.pw * (ki > ko ? ki : ko) < 0x7fffffffLL;
}

static size_t pack_bytes(int ki, int ko) {
    return static_cast<size_t>(ki / C) * (ko / C) * NFRAG * 64 * 16;
}

// How a layer is cut into workgroups (the same for every launch of the layer).
struct PatchPlan { int nh, nw, dchunk, nd; long long nblocks; bool pairs; int fold, fold_w; };
static PatchPlan plan_patches(const Geo &g, int ki, int ko) {
    PatchPlan p;
    const int nco = ko / C;
    // input channels in multiples of 64: two chunks per launch, summed on chip (4-row patches)
    p.pairs = ki % (2 * C) == 0;
    const int ph = p.pairs ? wide::PH : PH;
    // patches cover the largest output box of the grid (the interior grown on both sides)
    const int ed = g.td + 2 * grow_d(g), eh = g.th + 2 * g.grow, ew = g.tw + 2 * g.grow;
    p.nh = (eh + ph - 1) / ph;
    p.nw = (ew + PW - 1) / PW;
    // D chunk: whole box depth unless that leaves the chip short of workgroups
    const long long base = 1LL * g.ntiles * p.nh * p.nw * nco;
    int dchunk = ed;
    while (base * ((ed + dchunk - 1) / dchunk) < 1024 && dchunk > 16) dchunk = (dchunk + 1) / 2;
    // 2-D variant, tiles narrower than half a patch: up to 4 slices side by side (see fold_col); the tile's
    // slice count and the D chunk must be multiples of it
    p.fold = 1;
    p.fold_w = ew + 2;
    if (g.flat && 2 * (ew + 2) <= LCOLS) {
        int f = LCOLS / (ew + 2);
        if (f > 4) f = 4;
        while (f > 1 && g.td % f) --f;
        p.fold = f;
        dchunk = (dchunk + f - 1) / f * f;
    }
    p.dchunk = dchunk;
    p.nd = (ed + dchunk - 1) / dchunk;
    p.nblocks = base * p.nd;
    return p;
}

// workspace: packed weight fragments, then (layers that need more than one launch: more than one input
// chunk, or more than one pair of chunks when Cin is a multiple of 64) the fp32 partial sums: per workgroup
// and wave that stores results, dchunk planes x RH rows x 4 units x 1 KB (see part_unit)
size_t conv_mfma_ws_bytes(const Geo &g, int ki, int ko) {
    size_t n = pack_bytes(ki, ko);
    if (conv_gemm_preferred(g, ki, ko)) return n;      // one launch, sums stay in registers
    const PatchPlan p = plan_patches(g, ki, ko);
    const int launches = p.pairs ? ki / (2 * C) : ki / C;
    if (launches > 1)
        n += static_cast<size_t>(p.nblocks) * (p.pairs ? wide::NRG : kWaves) * p.dchunk * (RH * 4 * 256 * sizeof(float));
    return n;
}

bool conv_mfma_gather_supported(const Geo &g, int ki, int ko, sp_dtype_t dt) {
    // the marching kernels on a one-voxel margin, interiors only; per-lane offsets to the H / W neighbours (and
    // their sum at an edge) must fit the 32-bit staging offsets
    if (!conv_mfma_supported(g, ki, ko, dt) || g.halo != 1 || g.grow != 0 || g.flat || conv_gemm_preferred(g, ki, ko))
        return false;
    return static_cast<long long>(g.tile_vox) * (g.gw + 1) * (ki > ko ? ki : ko) < 0x7fffffffLL;
}

bool conv_mfma_bits_supported(const Geo &g, int ki, int ko, sp_dtype_t dt) {
    // the 3-D marching kernels (the wide-layer GEMM form and the 2-D variant keep the mask tensor)
    return conv_mfma_supported(g, ki, ko, dt) && !g.flat && !conv_gemm_preferred(g, ki, ko);
}

int launch_conv_mfma(const void *Pin, const void *w, const float *bias, void *Pout, const Geo &g,
                     int ki, int ko, bool relu, bool dgrad, void *ws, hipStream_t s, const void *mask,
                     const ConvSplit *split, bool gather, void *bits) {
    if (gather && !conv_mfma_gather_supported(g, ki, ko, SP_BF16)) return SP_EUNSUPPORTED;
    // one-bit mask: read by the data gradient in place of a mask tensor, written by a forward pass with ReLU
    if (bits && (!conv_mfma_bits_supported(g, ki, ko, SP_BF16) || (split && split->out2) || mask || (!dgrad && !relu)))
        return SP_EUNSUPPORTED;
    const int nci = ki / C, nco = ko / C;
    const int pack_elems = nci * nco * NFRAG * 64 * 8;
    hipLaunchKernelGGL(pack_weights_kernel, dim3((pack_elems + 255) / 256), dim3(256), 0, s,
                       static_cast<const uint16_t *>(w), static_cast<uint16_t *>(ws), ki, ko, dgrad ? 1 : 0, g.flat);
    int rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    // wide layers on few voxels: one launch that keeps the sums in registers over all input channels
    if (conv_gemm_preferred(g, ki, ko)) return launch_conv_gemm(Pin, ws, bias, Pout, g, ki, ko, relu, s, mask, split);
    ConvArgs a;
    a.in = static_cast<const uint16_t *>(Pin);
    a.bias = bias;
    a.out = static_cast<uint16_t *>(Pout);
    a.out2 = nullptr;
    a.out_ca = ko;
    a.out2_cs = 0;
    // two-tensor input: kernel channels [0, in_ca) come from Pin (in_ca per voxel), the rest from split->in2
    const uint16_t *in_a = static_cast<const uint16_t *>(Pin), *in_b = nullptr;
    int in_ca = ki;
    if (split && split->in2) {
        in_b = static_cast<const uint16_t *>(split->in2);
        in_ca = split->in_ca;
    }
    if (split && split->out2) {
        a.out2 = static_cast<uint16_t *>(split->out2);
        a.out_ca = split->out_ca;
        a.out2_cs = ko - split->out_ca;
    }
    // channels per voxel of the first output tensor (the whole output if there is no second one)
    const int out_cs_a = a.out2 ? a.out_ca : ko;
    a.mask = static_cast<const uint16_t *>(mask);
    a.bits = static_cast<uint16_t *>(bits);
    a.part = reinterpret_cast<float *>(static_cast<char *>(ws) + pack_bytes(ki, ko));
    a.g = g;
    a.out_cs = out_cs_a;
    a.nco = nco;
    // source of input chunk c (32 channels from channel 32 c of the concatenated input)
    auto chunk_src = [&](int cchunk, const uint16_t **base, int *cs, int *co) {
        const int c0 = C * cchunk;
        if (in_b && c0 >= in_ca) { *base = in_b; *cs = ki - in_ca; *co = c0 - in_ca; }
        else { *base = in_a; *cs = in_b ? in_ca : ki; *co = c0; }
    };
    const PatchPlan pl = plan_patches(g, ki, ko);
    const bool pairs = pl.pairs;
    a.nh = pl.nh;
    a.nw = pl.nw;
    a.dchunk = pl.dchunk;
    a.nd = pl.nd;
    a.fold = pl.fold;
    a.fold_w = pl.fold_w;
    a.gather = gather ? 1 : 0;
    const long long nb = pl.nblocks;
    if (nb > 0x7ffffff0LL) return SP_EGEOM;
    a.nblocks = static_cast<int>(nb);
    const unsigned grid = static_cast<unsigned>((nb + 7) / 8 * 8);
    using Kern = void (*)(ConvArgs);
    // [mode][bias][epilogue]; combinations that cannot occur (bias after the first launch, ReLU or mask before
    // the last, bias together with a mask) reuse the plain variant.  MB, RB: the two bit forms.
#define SP3D_TABLE(K, KD, MB, RB)                                                                          \
    {{{K<kSingle, false, kNone, KD>, K<kSingle, false, kRelu, KD>, K<kSingle, false, kMask, KD>,             \
       K<kSingle, false, MB, KD>, K<kSingle, false, RB, KD>},                                                \
      {K<kSingle, true, kNone, KD>, K<kSingle, true, kRelu, KD>, K<kSingle, false, kMask, KD>,               \
       K<kSingle, false, MB, KD>, K<kSingle, true, RB, KD>}},                                                \
     {{K<kFirst, false, kNone, KD>, K<kFirst, false, kNone, KD>, K<kFirst, false, kNone, KD>,                \
       K<kFirst, false, kNone, KD>, K<kFirst, false, kNone, KD>},                                            \
      {K<kFirst, true, kNone, KD>, K<kFirst, true, kNone, KD>, K<kFirst, true, kNone, KD>,                   \
       K<kFirst, true, kNone, KD>, K<kFirst, true, kNone, KD>}},                                             \
     {{K<kMiddle, false, kNone, KD>, K<kMiddle, false, kNone, KD>, K<kMiddle, false, kNone, KD>,             \
       K<kMiddle, false, kNone, KD>, K<kMiddle, false, kNone, KD>},                                          \
      {K<kMiddle, false, kNone, KD>, K<kMiddle, false, kNone, KD>, K<kMiddle, false, kNone, KD>,             \
       K<kMiddle, false, kNone, KD>, K<kMiddle, false, kNone, KD>}},                                         \
     {{K<kLast, false, kNone, KD>, K<kLast, false, kRelu, KD>, K<kLast, false, kMask, KD>,                   \
       K<kLast, false, MB, KD>, K<kLast, false, RB, KD>},                                                    \
      {K<kLast, false, kNone, KD>, K<kLast, false, kRelu, KD>, K<kLast, false, kMask, KD>,                   \
       K<kLast, false, MB, KD>, K<kLast, false, RB, KD>}}}
    // [2-D variant][mode][bias][epilogue]; the bit forms exist for the 3-D kernels only (the host refuses them
    // for 2-D geometries; their table entries repeat the plain kernel)
    static const Kern kern[2][4][2][5] = {SP3D_TABLE(conv_mfma_kernel, 3, kMaskBits, kReluBits),
                                          SP3D_TABLE(conv_mfma_kernel, 1, kNone, kNone)};
    static const Kern kern2[2][4][2][5] = {SP3D_TABLE(wide::conv_mfma_pair_kernel, 3, kMaskBits, kReluBits),
                                           SP3D_TABLE(wide::conv_mfma_pair_kernel, 1, kNone, kNone)};
#undef SP3D_TABLE
    const int epi = bits ? (dgrad ? kMaskBits : kReluBits) : (mask ? kMask : (relu ? kRelu : kNone));
    // more than 64 KB of dynamic LDS has to be requested explicitly
    static const hipError_t attr = [] {
        for (int i = 0; i < 80; ++i) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern[i / 40][(i / 10) & 3][(i / 5) & 1][i % 5]),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern2[i / 40][(i / 10) & 3][(i / 5) & 1][i % 5]),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, wide::LDS_BYTES);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }();
    if (attr != hipSuccess) return record_hip(attr);
    const int nsteps = pairs ? nci / 2 : nci;          // launches: input chunks, or pairs of them
    for (int ci = 0; ci < nsteps; ++ci) {
        const int mode = nsteps == 1 ? kSingle : (ci == 0 ? kFirst : (ci == nsteps - 1 ? kLast : kMiddle));
        chunk_src(pairs ? 2 * ci : ci, &a.in, &a.in_cs, &a.in_co);
        if (pairs) chunk_src(2 * ci + 1, &a.in2, &a.in2_cs, &a.in2_co);
        a.wpack = static_cast<const uint4 *>(ws) + static_cast<size_t>(pairs ? 2 * ci : ci) * nco * NFRAG * 64;
        if (pairs)
            hipLaunchKernelGGL(kern2[g.flat][mode][bias ? 1 : 0][epi], dim3(grid), dim3(kThreads), wide::LDS_BYTES, s, a);
        else
            hipLaunchKernelGGL(kern[g.flat][mode][bias ? 1 : 0][epi], dim3(grid), dim3(kThreads), LDS_BYTES, s, a);
        rc = record_hip(hipGetLastError());
        if (rc != SP_OK) return rc;
    }
    return SP_OK;
}

}  // namespace sp3d
