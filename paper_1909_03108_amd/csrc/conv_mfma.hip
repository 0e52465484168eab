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
#include "conv_mfma_common.h"

namespace sp3d {

using namespace convk;

namespace {

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
template <int P, bool EPI, int MODE, int RELU, bool FULL, int KD, int SIDE, int NV, bool HAS_BIAS>
__device__ __forceinline__ void plane_step(const Ctx<HAS_BIAS> &c, int Dp, int lane, const uint32_t (&lring)[2],
                                           const bf16x8 (&wf)[NFRAG], f32x16 (&acc)[4][RH],
                                           pin_t (&pin)[RH][4], mask_t (&mk)[RH][4],
                                           pin_t (&npin)[RH][4], mask_t (&nmk)[RH][4], bf16x8 (&b0)[RH + 2]) {
    constexpr int NR = RH + 2;
    constexpr int DONE = (P + 1) & 3;
    using S = Side<MODE, RELU, KD, false>;
    // ring slots of plane Dp and of plane Dp + 1, as a base register (slots 0, 1 / 2, 3) and an immediate that
    // fits the instruction's 16-bit offset field
    constexpr int PN = (P + 1) & 3;
    const uint32_t lbase = lring[P >> 1], lnext = lring[PN >> 1];
    constexpr int OFF = (P & 1) * PLANE_BYTES, OFFN = (PN & 1) * PLANE_BYTES;
    static_assert(PLANE_BYTES + 2 * CH_STRIDE + ((RH + 1) * LCOLS + 2) * 16 + CH_STRIDE < 65536, "offset field");
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
    for (int r = 0; r < NR; ++r) b[0][r] = b0[r];       // group 0's fragments: read, and waited for, by the previous step
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        const int kw = gi >> 1, half = gi & 1;
        if (gi + 1 < NG) {
            const int kw2 = (gi + 1) >> 1, half2 = (gi + 1) & 1;
#pragma unroll
            for (int r = 0; r < NR; ++r)
                frag_read(b[(gi + 1) & 1][r], lbase, OFF + half2 * 2 * CH_STRIDE + (r * LCOLS + kw2) * 16);
        } else {
            // The step's one synchronisation sits here, before its last group, not at its end: plane Dp + 1
            // must be complete (every wave's staging loads of it, issued two steps ago: loads complete in issue
            // order and the only ones issued after them are those of plane Dp + 2 and the NG - 1 of this step,
            // so "at most NV outstanding" implies it; stores share the counter and only make the wait more
            // conservative), and every wave must have finished reading plane Dp, this step's own (its last
            // fragment reads were issued a group ago; lgkmcnt(0) makes that formal), whose ring slot the next
            // step's staging loads overwrite.  Behind the barrier the first group of the NEXT step is read
            // already, while this step's last 18 MFMAs run: the step boundary itself has no wait, no barrier and
            // no exposed LDS latency.  (With the synchronisation at the end of the step the matrix cores idled
            // there for the barrier, the reads of two groups and their latency.)
            side_fence<NV, true, SIDE != kSideNone && S::PINS, SIDE != kSideNone && S::MASK,
                       SIDE != kSideNone && S::BITS>(npin, nmk);
            __builtin_amdgcn_s_barrier();
#pragma unroll
            for (int r = 0; r < NR; ++r) frag_read(b[0][r], lnext, OFFN + (r * LCOLS) * 16);
        }
        // this group's fragments were read a group ago; the NR reads issued just now may stay in flight
        frag_wait<NR>(b[gi & 1]);
        // keep the reads of the next group ahead of this group's MFMAs (the scheduler would
        // otherwise sink every read to just before its first use and expose the LDS latency)
        __builtin_amdgcn_sched_barrier(0);
        stage(c, Dp + DIST, gi, lane);
        if (gi < 4) {
            if (EPI) {
                // (the copies of the finished plane's sums out of the accumulation registers have no operand that
                // is computed in the step, so the compiler emits all 32 at the top of the step, in front of its
                // first MFMA; passing the plane through an empty statement here makes each group's eight depend
                // on a point inside the group, where they are woven between the MFMAs like the rest)
                asm volatile("" : "+a"(acc[DONE][0]), "+a"(acc[DONE][1]));
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
    // the next step's first fragments, read 18 MFMAs ago: complete before they leave the step (beyond it the
    // compiler may copy the registers at a block boundary, which it must not do while data is on its way)
    frag_wait<0>(b[0]);
#pragma unroll
    for (int r = 0; r < NR; ++r) b0[r] = b[0][r];
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
        if (KD == 3 && SP3D_PARKED(f)) park(wf[f]);
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

    // (the synchronisation of a step sits inside it, before its last MFMA group: see plane_step)
    constexpr int NV_STEP = (DIST - 1) * LOADS - 1;     // plane Dp + 2's loads and the step's first NG - 1
    static_assert(NG == LOADS, "one staging load per MFMA group");
    const uint32_t lring[2] = {lds_addr(lbase), lds_addr(lbase + 2 * PLANE_BYTES)};
    bf16x8 b0[RH + 2];
#pragma unroll
    for (int r = 0; r < RH + 2; ++r) b0[r] = *reinterpret_cast<const bf16x8 *>(lbase + (r * LCOLS) * 16);

    auto march = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        using S = Side<MODE, RELU, KD, false>;
        // whole patches fetch their partial sums / mask values one step ahead (see side_load): steps with an even
        // plane index use set A and fetch into set B, odd ones the other way round
        constexpr bool ASYNC = FULL && S::ASYNC;
        constexpr int FETCH = ASYNC ? kSideFetch : kSideNone, USE = ASYNC ? kSideUse : kSideNone;
        pin_t pinA[RH][4], pinB[RH][4];
        mask_t mkA[RH][4], mkB[RH][4];
        // (by its synchronisation point a step with stores has issued LOADS - 1 + 8 >= NV_STEP operations after its
        // side loads, so the wait covers them; the fetch-only step has issued just LOADS - 1 staging loads after
        // them and waits accordingly)
        static_assert(LOADS - 1 + 8 >= NV_STEP, "side loads must be older than what the step's wait lets stay in flight");
        // the first three steps have no finished plane to store (nplanes >= 3 always); the third one fetches
        // what the first store needs
        plane_step<0, false, MODE, RELU, FULL, KD, kSideNone, NV_STEP>(c, 0, lane, lring, wf, acc, pinA, mkA, pinB, mkB, b0);
        plane_step<1, false, MODE, RELU, FULL, KD, kSideNone, NV_STEP>(c, 1, lane, lring, wf, acc, pinA, mkA, pinB, mkB, b0);
        plane_step<2, false, MODE, RELU, FULL, KD, FETCH, (ASYNC ? LOADS - 1 : NV_STEP)>(c, 2, lane, lring, wf, acc, pinA,
                                                                                        mkA, pinB, mkB, b0);
        // steps 3, 4, 5, 6, 7, ...: planes mod 4 = 3, 0, 1, 2, 3, ...
#define SP3D_MAIN_STEP(OFF, PHASE, CP, CM, NP, NM)                                                            \
    if (D + (OFF) < nplanes)                                                                                  \
        plane_step<PHASE, true, MODE, RELU, FULL, KD, USE, NV_STEP>(c, D + (OFF), lane, lring, wf, acc, CP, CM, NP, NM, b0);
        for (int D = 3; D < nplanes; D += 4) {
            SP3D_MAIN_STEP(0, 3, pinB, mkB, pinA, mkA)
            SP3D_MAIN_STEP(1, 0, pinA, mkA, pinB, mkB)
            SP3D_MAIN_STEP(2, 1, pinB, mkB, pinA, mkA)
            SP3D_MAIN_STEP(3, 2, pinA, mkA, pinB, mkB)
        }
#undef SP3D_MAIN_STEP
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
}

}  // namespace


bool conv_mfma_supported(const Geo &g, int ki, int ko, sp_dtype_t dt) {
    // per-lane staging offsets inside a padded plane are 32-bit: element offsets in the one-chunk kernel, byte
    // offsets in the two-chunk kernel (input channels in multiples of 64)
    const long long lim = ki % (2 * C) == 0 ? 0x3fffffffLL : 0x7fffffffLL;
    return dt == SP_BF16 && ki % C == 0 && ko % C == 0 && ki <= 1024 && ko <= 1024 &&
           1LL * g.ph * g.pw * (ki > ko ? ki : ko) < lim;
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
    const long long lim = ki % (2 * C) == 0 ? 0x3fffffffLL : 0x7fffffffLL;       // see conv_mfma_supported
    return static_cast<long long>(g.tile_vox) * (g.gw + 1) * (ki > ko ? ki : ko) < lim;
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
    // [2-D variant][mode][bias][epilogue]; the bit forms exist for the 3-D kernels only (the host refuses them
    // for 2-D geometries; their table entries repeat the plain kernel).  The two-chunk kernels have the same table
    // in their own translation unit (conv_mfma_pair.hip).
    static const Kern kern[2][4][2][5] = {SP3D_CONV_TABLE(conv_mfma_kernel, 3, kMaskBits, kReluBits),
                                          SP3D_CONV_TABLE(conv_mfma_kernel, 1, kNone, kNone)};
    const int epi = bits ? (dgrad ? kMaskBits : kReluBits) : (mask ? kMask : (relu ? kRelu : kNone));
    // more than 64 KB of dynamic LDS has to be requested explicitly
    static const hipError_t attr = [] {
        for (int i = 0; i < 80; ++i) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern[i / 40][(i / 10) & 3][(i / 5) & 1][i % 5]),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
            if (e != hipSuccess) return e;
        }
        return conv_mfma_pair_prepare();
    }();
    if (attr != hipSuccess) return record_hip(attr);
    const int nsteps = pairs ? nci / 2 : nci;          // launches: input chunks, or pairs of them
    for (int ci = 0; ci < nsteps; ++ci) {
        const int mode = nsteps == 1 ? kSingle : (ci == 0 ? kFirst : (ci == nsteps - 1 ? kLast : kMiddle));
        chunk_src(pairs ? 2 * ci : ci, &a.in, &a.in_cs, &a.in_co);
        if (pairs) chunk_src(2 * ci + 1, &a.in2, &a.in2_cs, &a.in2_co);
        a.wpack = static_cast<const uint4 *>(ws) + static_cast<size_t>(pairs ? 2 * ci : ci) * nco * NFRAG * 64;
        if (pairs)
            conv_mfma_pair_launch(g.flat, mode, bias ? 1 : 0, epi, grid, s, a);
        else
            hipLaunchKernelGGL(kern[g.flat][mode][bias ? 1 : 0][epi], dim3(grid), dim3(kThreads), LDS_BYTES, s, a);
        rc = record_hip(hipGetLastError());
        if (rc != SP_OK) return rc;
    }
    return SP_OK;
}

}  // namespace sp3d
