// Shared by conv_mfma.hip (one input chunk per launch) and conv_mfma_pair.hip (two): operand layouts, kernel
// arguments, epilogue pieces.  See conv_mfma.hip for the design.
#pragma once
#include "common.h"

#include <type_traits>

namespace sp3d {
namespace convk {


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

// two floats -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack2(float a, float b) {
    union { bf16x2 v; uint32_t u; } r;
    r.v = __builtin_convertvector(f32x2{a, b}, bf16x2);
    return r.u;
}

// The 54 weight fragments of a lane (216 registers) do not fit beside everything else in the 256 ordinary vector
// registers, and what the compiler evicts to the accumulation half of the register file it copies back before
// every use (two thirds of all copies between the halves in the plane step, a quarter of its instructions).  The
// matrix instructions read their A operand from either half: a fragment that passes through here is defined in
// the accumulation half and is used from there, with no copy.
#ifndef SP3D_PARKED
#define SP3D_PARKED(f) ((f) % 3 == 0)
#endif
__device__ __forceinline__ void park(bf16x8 &w) { asm volatile("" : "+a"(w)); }

// LDS fragment reads by hand.  The compiler counts a direct-to-LDS load as an access of both memories, and
// while one is in flight - here: always - it turns every wait for an LDS read into "all LDS reads done"
// (s_waitcnt lgkmcnt(0)).  In the plane step that wait stands behind the reads of the NEXT group, issued a moment
// earlier, so each of the six groups began by sitting out a full LDS latency with idle matrix cores.  LDS reads
// return in issue order: "at most NR outstanding" is all a group needs, and that is what frag_wait states; the
// registers pass through it as operands, so nothing uses them earlier.
__device__ __forceinline__ void frag_read(bf16x8 &d, uint32_t base, int off) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(base), "i"(off) : "memory");
}
// LDS address (the 32-bit offset that the instructions take) of a pointer into the dynamic LDS block
__device__ __forceinline__ uint32_t lds_addr(const char *p) {
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) char *)p));
}
template <int N>
__device__ __forceinline__ void frag_wait(bf16x8 (&f)[4]) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : "n"(N) : "memory");
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
// patches, whose loads are predicated, keep the ordinary loads.  Between a side load and the wait that covers it
// the code must be one basic block with nothing that makes the compiler move the register: a load issued under
// a run-time condition is joined to the other path by a copy that runs before the data has arrived.
__device__ __forceinline__ void side_load(pin_t &d, const float *p) {
    // (partial sums: a contiguous kilobyte per wave, read once - non-temporal)
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(d) : "v"(p) : "memory");
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
// Measured: the mask gains from them (3-D 32 -> 32 at 512^3: 7.45 -> 7.08 ms; 2-D: 8 - 9 %; the 3-D two-chunk
// kernel 3 %, now that part of its weight fragments live in LDS - while its registers were all taken the second
// register set cost 4.07 -> 4.71 ms).  Partial sums: ordinary loads in the one-chunk kernel; in the two-chunk
// kernel a wave finishes one row of its two (conv_mfma_pair_kernel.h) and has room for a second set of that row's
// 16 registers.  (While one wave finished both rows, the second set of 32 registers spilled, and the reloads
// wait on the same counter: 4 % slower than ordinary loads, which cost 35 - 45 % of the cycles of a launch.)
template <int MODE, int RELU, int KD, bool PAIR> struct Side {
    static constexpr bool PINS = MODE == kMiddle || MODE == kLast;
    static constexpr bool MASK = (RELU == kMask || RELU == kMaskBits) && (MODE == kSingle || MODE == kLast);
    static constexpr bool BITS = MASK && RELU == kMaskBits;      // one 16-bit word per row instead of 4 x 8 bytes
    static constexpr bool ASYNC = MASK && !PINS;
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

// ReLU on the bit pattern of an fp32 value: whatever has the sign bit set (negative values, -0, NaNs with the sign
// set) becomes +0, everything else stays as it is - one integer maximum, where the floating-point compare and select
// (which keeps every NaN) cost two instructions and the two idle cycles the select waits for the compare's result.
__device__ __forceinline__ float relu_f32(float v) { return __int_as_float(max(__float_as_int(v), 0)); }

// The mask bit of a ReLU result v (sign clear), shifted into `word` from the right.  Taken from the fp32 value before
// it is rounded: a value is stored as a positive bf16 exactly if it exceeds 2^-134 (pattern 0x00008000), the midpoint
// between zero and the smallest bf16 denormal (a tie rounds to the even neighbour, zero; fp32 denormals are kept in
// these kernels' floating-point mode), and for patterns with a clear sign the integer order is the floating-point
// order: 0x8000 - pattern is negative exactly then (+inf included; a NaN, which ReLU leaves only with a clear sign,
// counts as positive here, while the stand-alone bit kernel gives it a zero bit).  One subtraction and one funnel
// shift per value and no compare: the compare-and-select form cost two instructions, two idle cycles and the OR.
__device__ __forceinline__ uint32_t shift_in_positive(uint32_t word, float v) {
    return __builtin_amdgcn_alignbit(word, static_cast<uint32_t>(0x8000 - __float_as_int(v)), 31);
}
// After the row's 16 values went in, in the order k = 4 q + i, bit 15 - k holds value k: reverse.
__device__ __forceinline__ uint16_t row_word(uint32_t shifted) {
    return static_cast<uint16_t>(__builtin_bitreverse32(shifted) >> 16);
}
// ... and the reverse, for the reader.  spread_word, once per row: the row's word in the low half and the word
// shifted right by one in the high half, so that bits k and k + 1 (k even) sit at position k of the two halves.
// nibble_halves, per store unit q: 0xffff in each half of the unit's two packed words whose bit is set - a packed
// shift that brings position 4 q (4 q + 2 for the second word) of both halves to their sign bits and a packed
// arithmetic shift that fills the halves with it.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t spread_word(uint32_t word) { return ((word >> 1) << 16) | (word & 0xffffu); }
__device__ __forceinline__ uint32_t fill_from_bit(uint32_t spread, int k) {
    union { uint32_t u; u16x2 v; s16x2 s; } r;
    r.u = spread;
    r.v = r.v << static_cast<unsigned short>(15 - k);
    r.s = r.s >> static_cast<short>(15);
    return r.u;
}
__device__ __forceinline__ uint2 nibble_halves(uint32_t spread, int q) {
    return make_uint2(fill_from_bit(spread, 4 * q), fill_from_bit(spread, 4 * q + 2));
}

// kReluBits: write the mask word of row h of plane d that the four store units of the row collected.
template <bool FULL, class CtxT>
__device__ __forceinline__ void store_bits(const CtxT &c, int d, const mask_t (&mk)[RH][4], int h) {
    if (FULL || c.okrow[h]) c.bbase[bits_off(c, d, h)] = row_word(mk[h][0].x);
}

// ---- the two-chunk kernel (conv_mfma_pair.hip) ------------------------------------------------
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

}  // namespace wide

}  // namespace convk

// Kernel table of a family K<mode, bias, epilogue, KD>: [mode][bias][epilogue]; combinations that cannot occur
// (bias after the first launch, ReLU or mask before the last, bias together with a mask) reuse the plain variant.
// MB, RB: the two bit forms of the epilogue (or kNone where a family does not have them).
#define SP3D_CONV_TABLE(K, KD, MB, RB)                                                                          \
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

// conv_mfma_pair.hip: the kernels of namespace wide.  [2-D variant][mode][bias][epilogue], see launch_conv_mfma.
hipError_t conv_mfma_pair_prepare();      // requests the dynamic LDS of every variant (once)
void conv_mfma_pair_launch(int flat, int mode, int bias, int epi, unsigned grid, hipStream_t s,
                           const convk::ConvArgs &a);

}  // namespace sp3d
