// The two-chunk form of the plane-marching convolution kernel (see conv_mfma.hip for the single-chunk form and
// the common design).  Included by conv_mfma_pair.hip (3-D kernels) and conv_mfma_pair2d.hip (2-D variant), which
// instantiate one half of the kernel table each, so that the two halves compile side by side.
// Two input chunks per launch (layers with Cin a multiple of 64).  With one chunk per launch every extra
// chunk costs a round trip of the fp32 partial sums through HBM (8 bytes per output value), which makes
// wide layers bandwidth-bound.  Here a workgroup contracts 64 input channels at once and adds the two
// halves on chip: the patch is 4 rows x 32 columns, waves 0, 1 take input chunk 0 and waves 2, 3 chunk 1
// of the pair, each for one row group of 2 rows, with the same register-resident weights, D march and
// fragment reuse as above.  The two waves with the same rows (one per chunk) share the epilogue by rows: when an
// output plane is complete, each writes the accumulators of ONE of its two rows to a small LDS buffer (during
// the next step, between its MFMAs); one step later, after the step barrier, the other adds them to its own,
// converts and stores - the chunk-0 wave finishes row 0, the chunk-1 wave row 1.  A plane therefore lives in
// an accumulator slot for five steps (three contributing, one being handed over, one being stored), hence
// five slots.  Layers with more than one pair still go through fp32 partial sums, but half as often.
#pragma once
#include "conv_mfma_common.h"

namespace sp3d {

namespace convk {
namespace wide {      // (inside the namespace of its constants: LOADS, PLANE_BYTES, ... mean the two-chunk kernel's)

// direct-to-LDS load as in wgrad_mfma.hip: written as assembly so that the compiler neither tracks it nor
// drains it before unrelated LDS accesses; the kernel counts the loads itself (s_waitcnt vmcnt)
// Address = uniform base (scalar registers) + this lane's unsigned 32-bit byte offset: one register per staging
// load instead of a 64-bit pair, and no per-load address arithmetic.  Offsets can be negative (gathered halos
// point into a neighbour tile), so they are kept with a bias of 2^31 that the base takes back.
constexpr uint32_t kOffBias = 0x80000000u;
__device__ __forceinline__ void dma16(const uint16_t *base, uint32_t off, const char *dst) {
    const uint32_t l = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (const __attribute__((address_space(3))) char *)dst));
    const char *b = reinterpret_cast<const char *>(base) - static_cast<ptrdiff_t>(kOffBias);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(b), "s"(l) : "memory");
}

template <bool HAS_BIAS>
struct Ctx {
    const uint16_t *tin0;       // first padded input plane of the D chunk, at this wave's input chunk
    size_t plane_elems;
    int nplanes;
    int plo, phi;               // staged planes are clamped to [plo, phi]
    ptrdiff_t dlo, dhi;         // gathered halos: what to add for staged plane 0 / the last one (else 0)
    uint32_t goff[LOADS];       // source offsets of the staging loads (bytes, biased by kOffBias)
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
    if (j % CP_LOADS != CP_LOADS - 1 || c.tail_lane) dma16(p, c.goff[j], dst);
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

// what the partner wrote for store unit q of row h (see give_unit)
__device__ __forceinline__ float4 handed_over(const char *red, int h, int q) {
    return *reinterpret_cast<const float4 *>(red + (h * 4 + q) * 1024);
}
// finish 4 channels of row h of plane d: (own sum + what the partner handed over, from LDS) + the earlier pairs'
// partial sums in the launches after a layer's first, then store the new partial (fp32) or ReLU / convert / store
// bf16.  The order of the additions is the same whichever of the two waves finishes the row: a voxel that two
// tiles both compute (a block of layers after one exchange) may be in row 0 in one and in row 1 in the other, and
// has to come out with the same bits.
// (o: what handed_over read for this unit)
template <int MODE, int RELU, bool FULL, bool HAS_BIAS>
__device__ __forceinline__ void finish_unit(const Ctx<HAS_BIAS> &c, int d, const f32x16 (&s)[RH], const float4 &o,
                                            const pin_t (&pin)[RH][4], mask_t (&mk)[RH][4], int h, int q) {
    float v0 = s[h][4 * q] + o.x, v1 = s[h][4 * q + 1] + o.y, v2 = s[h][4 * q + 2] + o.z, v3 = s[h][4 * q + 3] + o.w;
    if (MODE == kMiddle || MODE == kLast) { v0 += pin[h][q].x; v1 += pin[h][q].y; v2 += pin[h][q].z; v3 += pin[h][q].w; }
    const size_t at = d * c.oplane + h * c.orow + 8 * q;
    if (MODE == kFirst || MODE == kMiddle) {
        // (a contiguous kilobyte per wave that the next launch reads once: non-temporal)
        if (FULL || c.okrow[h])
            __builtin_nontemporal_store(pin_t{v0, v1, v2, v3}, reinterpret_cast<pin_t *>(c.pbase + part_unit(d, h, q)));
        return;
    }
    if (is_relu(RELU)) {
        v0 = relu_f32(v0); v1 = relu_f32(v1); v2 = relu_f32(v2); v3 = relu_f32(v3);
    }
    uint2 pk = make_uint2(pack2(v0, v1), pack2(v2, v3));
    if (RELU == kMask) {
        pk.x &= positive_halves(mk[h][q].x);
        pk.y &= positive_halves(mk[h][q].y);
    }
    if (RELU == kMaskBits) {
        if (q == 0) mk[h][0].x = spread_word(mk[h][0].x);
        const uint2 m = nibble_halves(mk[h][0].x, q);
        pk.x &= m.x;
        pk.y &= m.y;
    }
    if (FULL || c.okrow[h]) *reinterpret_cast<uint2 *>(c.obase + at) = pk;
    if (RELU == kReluBits) {
        // the row's word collects in the (otherwise unused) mask register of unit 0 and leaves with the last unit
        uint32_t n = mk[h][0].x;
        n = shift_in_positive(n, v0); n = shift_in_positive(n, v1);
        n = shift_in_positive(n, v2); n = shift_in_positive(n, v3);
        mk[h][0].x = n;
        if (q == 3) store_bits<FULL>(c, d, mk, h);
    }
}

// hand 4 channels of row h of a complete plane over to the partner
__device__ __forceinline__ void give_unit(const f32x16 (&s)[RH], char *red, int h, int q) {
    *reinterpret_cast<float4 *>(red + (h * 4 + q) * 1024) =
        make_float4(s[h][4 * q], s[h][4 * q + 1], s[h][4 * q + 2], s[h][4 * q + 3]);
}

// The wait of a step (NV vector-memory operations may stay outstanding, LDS operations none) with one row's side
// registers as operands (see side_fence): the partial sums of the row the wave hands over, the mask values - or,
// in the bit form, the one word kept in m[0].x - of the row it finishes.
template <int NV, bool PINS, bool MASK, bool BITS>
__device__ __forceinline__ void side_fence_row(pin_t (&p)[4], mask_t (&m)[4]) {
    static_assert(!(MASK && BITS), "one form of the mask");
#define SP3D_ROW4(a) "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])
    if (PINS && MASK) asm volatile("s_waitcnt vmcnt(%8) lgkmcnt(0)" : SP3D_ROW4(p), SP3D_ROW4(m) : "n"(NV) : "memory");
    else if (PINS && BITS) asm volatile("s_waitcnt vmcnt(%5) lgkmcnt(0)" : SP3D_ROW4(p), "+v"(m[0].x) : "n"(NV) : "memory");
    else if (PINS) asm volatile("s_waitcnt vmcnt(%4) lgkmcnt(0)" : SP3D_ROW4(p) : "n"(NV) : "memory");
    else if (MASK) asm volatile("s_waitcnt vmcnt(%4) lgkmcnt(0)" : SP3D_ROW4(m) : "n"(NV) : "memory");
    else if (BITS) asm volatile("s_waitcnt vmcnt(%1) lgkmcnt(0)" : "+v"(m[0].x) : "n"(NV) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NV) : "memory");
#undef SP3D_ROW4
}

// One staged input plane Dp.  P = Dp mod 5: output plane Dp - kd accumulates in slot (P - kd) mod 5.
// The epilogue of the pair's 2 x 2 rows is shared by rows: the wave of chunk ROLE finishes row ROLE of its row
// group and hands row 1 - ROLE over to its partner (the wave of the other chunk with the same rows).
// GIVE: row 1 - ROLE of plane Dp - 3 (slot (P + 2) mod 5) goes to the hand-over buffer Dp & 1.  FIN: row ROLE of
// plane Dp - 4 (slot (P + 1) mod 5) is finished with what the partner wrote in the previous step, buffer
// (Dp - 1) & 1, and - in the launches after a layer's first - the earlier pairs' partial sums.  A slot returns
// to the bias (chunk 0) or zero (chunk 1) when it becomes the slot of plane Dp + 1.  (With all the finishing on
// the chunk-0 wave and all the handing over on the chunk-1 wave, a step lasted as long as the former's epilogue.)
// SIDE (see side_load): the partial sums and mask values of the row that the NEXT step finishes (plane Dp - 3)
// are fetched at the start of this step into the other register set (npin, nmk) and pass through the step's
// wait; the step itself uses what the previous one fetched (pin, mk).  Without it the step loads what it needs
// the ordinary way.
// lcur / lnxt: this lane's LDS read base in the ring slots of planes Dp / Dp + 1; b0: the fragments of the first
// MFMA group, read (and waited for) by the previous step; on return those of the next step.  NV: how many
// vector-memory operations the step's wait, which stands before its last MFMA group, lets stay in flight.
template <int P, int ROLE, bool GIVE, bool FIN, int MODE, int RELU, bool FULL, int KD, bool SIDE, int NV, bool HAS_BIAS>
__device__ __forceinline__ void plane_step(const Ctx<HAS_BIAS> &c, int Dp, uint32_t lcur, uint32_t lnxt,
                                           const bf16x8 (&wf)[NFRAG], f32x16 (&acc)[NSLOT][RH],
                                           pin_t (&pin)[RH][4], mask_t (&mk)[RH][4],
                                           pin_t (&npin)[RH][4], mask_t (&nmk)[RH][4], bf16x8 (&b0)[RH + 2]) {
    constexpr int NR = RH + 2;
    static_assert(NR == 4, "frag_wait names four fragments");
    static_assert(RH == 2, "one row to finish, one to hand over");
    static_assert(2 * CH_STRIDE + ((RH + 1) * LCOLS + 2) * 16 < 65536, "offset field of the LDS reads");
    constexpr int FROW = ROLE, GROW = 1 - ROLE;      // the row this wave finishes / hands over
    constexpr int GSLOT = (P + 2) % NSLOT, FSLOT = (P + 1) % NSLOT;
    constexpr int NEXT = (P + 1) % NSLOT;      // slot of output plane Dp + 1: must be clean when this step ends
    using S = Side<MODE, RELU, KD, true>;
    bf16x8 b[2][NR];
    char *red_w = c.red + (Dp & 1) * RED_BYTES;
    const char *red_r = c.red + ((Dp - 1) & 1) * RED_BYTES;
    if (SIDE) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const size_t at = (Dp - 3) * c.oplane + FROW * c.orow + 8 * q;
            if (S::PINS) side_load(npin[FROW][q], c.pbase + part_unit(Dp - 3, FROW, q));
            if (S::MASK && !S::BITS) side_load(nmk[FROW][q], c.mbase + at);
            if (S::BITS && q == 0) SP3D_SIDE_LOAD_BITS(nmk[FROW][0].x, c.bbase + bits_off(c, Dp - 3, FROW));
        }
    }
    if (!SIDE && FIN) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (S::PINS) pin[FROW][q] = load_partial<FULL>(c, Dp - 4, FROW, q);
            if (S::MASK) mk[FROW][q] = load_mask<FULL, S::BITS>(c, Dp - 4, FROW, q);
        }
    }
#pragma unroll
    for (int r = 0; r < NR; ++r) b[0][r] = b0[r];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        const int kw = gi >> 1, half = gi & 1;
        if (gi + 1 < NG) {
            const int kw2 = (gi + 1) >> 1, half2 = (gi + 1) & 1;
#pragma unroll
            for (int r = 0; r < NR; ++r)
                frag_read(b[(gi + 1) & 1][r], lcur, half2 * 2 * CH_STRIDE + (r * LCOLS + kw2) * 16);
        } else {
            // The step's synchronisation stands here, before its last MFMA group (see the one-chunk kernel's
            // plane_step): plane Dp + 1 has landed when at most the loads of plane Dp + 2 and this step's first
            // LOADS - 1 are in flight; this wave's hand-over writes (issued in groups 0 - 3) have reached LDS and
            // its reads of plane Dp and of the other role's hand-over are done (lgkmcnt(0)).  Behind the barrier
            // the first group of the next step is read while this step's last 18 MFMAs run.
            side_fence_row<NV, SIDE && S::PINS, SIDE && S::MASK && !S::BITS, SIDE && S::BITS>(npin[FROW], nmk[FROW]);
            __builtin_amdgcn_s_barrier();
#pragma unroll
            for (int r = 0; r < NR; ++r) frag_read(b[0][r], lnxt, (r * LCOLS) * 16);
        }
        // this group's fragments were read a group ago; the NR reads issued just now may stay in flight
        frag_wait<NR>(b[gi & 1]);
        // the two weight fragments of this group that live in LDS (see WL_FRAGS); the MFMAs that use them are
        // the last of the group
        // ... and what the partner handed over for this group's store unit: read here, at the top of the group, six
        // and more MFMAs before the first addition that needs it
        float4 ho = make_float4(0.f, 0.f, 0.f, 0.f);
        if (FIN && gi < 4) ho = handed_over(red_r, FROW, gi);
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
            // (the empty statements tie the copies out of the accumulation registers to this group; otherwise the
            // compiler emits all of them at the top of the step, in front of its first MFMA)
            if (GIVE) {
                asm volatile("" : "+a"(acc[GSLOT][GROW]));
                give_unit(acc[GSLOT], red_w, GROW, gi);
            }
            if (FIN) {
                asm volatile("" : "+a"(acc[FSLOT][FROW]));
                finish_unit<MODE, RELU, FULL>(c, Dp - 4, acc[FSLOT], ho, pin, mk, FROW, gi);
            }
        } else {
            // the slot of the next output plane starts from the bias (chunk 0) or zero (chunk 1); in the first
            // steps it holds sums for planes that do not exist
#pragma unroll
            for (int i = 0; i < 16; ++i)
                acc[NEXT][gi - 4][i] = (ROLE == 0 && HAS_BIAS) ? c.bv[HAS_BIAS ? i : 0] : 0.f;
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
    // the next step's first fragments, read 18 MFMAs ago: complete before they leave the step
    frag_wait<0>(b[0]);
#pragma unroll
    for (int r = 0; r < NR; ++r) b0[r] = b[0][r];
}

// The two steps after the last input plane: only the side work is left.  Dp = nplanes: the last output plane
// (Dp - 3 = dn - 1) is handed over and plane Dp - 4 finished; Dp = nplanes + 1: the last plane is finished.  Same
// slot arithmetic as plane_step, so every accumulator index stays a constant.
template <int P, int ROLE, bool GIVE, bool FIN, int MODE, int RELU, bool FULL, int KD, bool SIDE, bool HAS_BIAS>
__device__ __forceinline__ void drain_step(const Ctx<HAS_BIAS> &c, int Dp, f32x16 (&acc)[NSLOT][RH],
                                           pin_t (&pin)[RH][4], mask_t (&mk)[RH][4],
                                           pin_t (&npin)[RH][4], mask_t (&nmk)[RH][4]) {
    constexpr int FROW = ROLE, GROW = 1 - ROLE;
    constexpr int GSLOT = (P + 2) % NSLOT, FSLOT = (P + 1) % NSLOT;
    using S = Side<MODE, RELU, KD, true>;
    if (GIVE && Dp == c.nplanes) {
        char *red_w = c.red + (Dp & 1) * RED_BYTES;
#pragma unroll
        for (int q = 0; q < 4; ++q) give_unit(acc[GSLOT], red_w, GROW, q);
    }
    // Side loads for the step after this one, like a plane step's (a drain step can be step 3 already: a march of
    // three planes).  From here to the wait that follows the step the code is one straight line: a register with
    // a load in flight must not meet a block boundary, where the compiler may copy it.  Hence no condition on the
    // second drain step, which needs nothing: it fetches the last plane's values once more.
    if (SIDE) {
        const int dl = min(Dp - 3, c.nplanes - 3);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const size_t at = dl * c.oplane + FROW * c.orow + 8 * q;
            if (S::PINS) side_load(npin[FROW][q], c.pbase + part_unit(dl, FROW, q));
            if (S::MASK && !S::BITS) side_load(nmk[FROW][q], c.mbase + at);
            if (S::BITS && q == 0) SP3D_SIDE_LOAD_BITS(nmk[FROW][0].x, c.bbase + bits_off(c, dl, FROW));
        }
    }
    if (FIN) {
        const char *red_r = c.red + ((Dp - 1) & 1) * RED_BYTES;
        if (!SIDE) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (S::PINS) pin[FROW][q] = load_partial<FULL>(c, Dp - 4, FROW, q);
                if (S::MASK) mk[FROW][q] = load_mask<FULL, S::BITS>(c, Dp - 4, FROW, q);
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
            finish_unit<MODE, RELU, FULL>(c, Dp - 4, acc[FSLOT], handed_over(red_r, FROW, q), pin, mk, FROW, q);
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
                if (KD == 3 && SP3D_PARKED(f)) park(wf[f]);
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
    int goff[LOADS];            // in elements; the host has checked that twice their value fits 32 bits
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int v = 64 * (j % CP_LOADS) + lane;
        const FoldCol fc = fold_col(v % LCOLS, F, a.fold_w);
        const int row = min(h0 + v / LCOLS, bx.bh + 1), colv = min(w0 + fc.c, bx.bw + 1);
        goff[j] = ((min(fc.s, F - 1) * g.ph + row) * g.pw + colv) * src_cs + (2 * rg + j / CP_LOADS) * 8;   // always addressable
    }
    c.dlo = c.dhi = 0;
    if (a.gather) {          // see GatherShift
        const GatherShift gs = gather_shift(g, tile, src_cs);
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const int v = 64 * (j % CP_LOADS) + lane;
            const int row = min(h0 + v / LCOLS, bx.bh + 1), colv = min(w0 + v % LCOLS, bx.bw + 1);
            goff[j] += (row == 0 ? gs.hm : 0) + (row == g.th + 1 ? gs.hp : 0) + (colv == 0 ? gs.wm : 0) +
                       (colv == g.tw + 1 ? gs.wp : 0);
        }
        if (d0 == 0) c.dlo = gs.dm;
        if (d0 + dn == g.td) c.dhi = gs.dp;
    }
#pragma unroll
    for (int j = 0; j < LOADS; ++j) c.goff[j] = static_cast<uint32_t>(goff[j] * 2) + kOffBias;
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
    // row group rg of workgroup `logical` (both of its waves): dchunk planes x RH rows x 4 units x 1 KB
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

    // (a plane step synchronises inside itself, before its last MFMA group; a drain step at its end)
    constexpr int NV_STEP = (DIST - 1) * LOADS - 1;     // plane Dp + 2's loads and the step's first LOADS - 1
    const uint32_t lring = lds_addr(lbase);
    bf16x8 b0[RH + 2];
#pragma unroll
    for (int r = 0; r < RH + 2; ++r) b0[r] = *reinterpret_cast<const bf16x8 *>(lbase + (r * LCOLS) * 16);

    auto march = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        using S = Side<MODE, RELU, KD, true>;
        // whole patches: each wave fetches the partial sums and mask values of the row it finishes one step ahead
        // (see side_load), alternating between two sets of registers.  Step 4 is the first to finish a row, so
        // step 3 is the first to fetch.
        constexpr bool SD = FULL && (S::PINS || S::MASK);
        pin_t pinA[RH][4], pinB[RH][4];
        mask_t mkA[RH][4], mkB[RH][4];
        // By its wait a step has issued LOADS - 1 staging loads after its side loads, and four stores if it
        // finishes a row: that many operations the wait may let stay in flight (never more than NV_STEP, which
        // is what it takes for plane Dp + 1 to have landed).  A drain step issues no staging loads and waits for
        // everything.
        static_assert(LOADS - 1 + 4 <= NV_STEP, "a wait that covers the side loads covers the staged plane");
#define SP3D_NV_OF(SIDES, FIN_EN) ((SIDES) ? LOADS - 1 + ((FIN_EN) ? 4 : 0) : NV_STEP)
        plane_step<0, ROLE, false, false, MODE, RELU, FULL, KD, false, NV_STEP>(
            c, 0, lring, lring + PLANE_BYTES, wf, acc, pinA, mkA, pinB, mkB, b0);
        plane_step<1, ROLE, false, false, MODE, RELU, FULL, KD, false, NV_STEP>(
            c, 1, lring + PLANE_BYTES, lring + 2 * PLANE_BYTES, wf, acc, pinA, mkA, pinB, mkB, b0);
        plane_step<2, ROLE, false, false, MODE, RELU, FULL, KD, false, NV_STEP>(
            c, 2, lring + 2 * PLANE_BYTES, lring + 3 * PLANE_BYTES, wf, acc, pinB, mkB, pinA, mkA, b0);
        // Steps 3, 4, ... with slot phase Dp mod 5 as a compile-time constant (the ring slot Dp mod 4 is a
        // run-time offset: a period of 20 steps would be needed to make both constants).  The march runs two
        // steps past the last input plane; those only hand over / finish what is left.  Step 3 is the first
        // to hand a row over, step 4 the first to finish one.
#define SP3D_STEP(DP, PHASE, FIN_EN, CP, CM, NP, NM)                                                       \
    if ((DP) < nplanes) {                                                                                  \
        plane_step<PHASE, ROLE, true, FIN_EN, MODE, RELU, FULL, KD, SD, SP3D_NV_OF(SD, FIN_EN)>(           \
            c, (DP), lring + ((DP) % NBUF) * PLANE_BYTES, lring + (((DP) + 1) % NBUF) * PLANE_BYTES, wf, acc, CP, CM, \
            NP, NM, b0);                                                                                   \
    } else if ((DP) < nplanes + 2) {                                                                       \
        drain_step<PHASE, ROLE, true, FIN_EN, MODE, RELU, FULL, KD, SD>(c, (DP), acc, CP, CM, NP, NM);     \
        side_fence_row<(SD ? 0 : (DIST - 1) * LOADS), SD && S::PINS, SD && S::MASK && !S::BITS, SD && S::BITS>( \
            NP[ROLE], NM[ROLE]);                                                                           \
        __builtin_amdgcn_s_barrier();                                                                      \
    }
        SP3D_STEP(3, 3, false, pinA, mkA, pinB, mkB)
        SP3D_STEP(4, 4, true, pinB, mkB, pinA, mkA)
        for (int D = 5; D < nplanes + 2; D += NSLOT) {
            SP3D_STEP(D, 0, true, pinA, mkA, pinB, mkB)
            SP3D_STEP(D + 1, 1, true, pinB, mkB, pinA, mkA)
            SP3D_STEP(D + 2, 2, true, pinA, mkA, pinB, mkB)
            SP3D_STEP(D + 3, 3, true, pinB, mkB, pinA, mkA)
            SP3D_STEP(D + 4, 4, true, pinA, mkA, pinB, mkB)
            // five steps per round: the sets have changed roles
            if (SD) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const pin_t tp = pinA[ROLE][q]; pinA[ROLE][q] = pinB[ROLE][q]; pinB[ROLE][q] = tp;
                    const mask_t tm = mkA[ROLE][q]; mkA[ROLE][q] = mkB[ROLE][q]; mkB[ROLE][q] = tm;
                }
            }
        }
#undef SP3D_STEP
#undef SP3D_NV_OF
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // clamped staging loads of the last steps
    };
    if (h0 + PH <= bx.bh && w0 + PW <= bx.bw) march(std::true_type{});
    else march(std::false_type{});
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
}  // namespace convk

}  // namespace sp3d
