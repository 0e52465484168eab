// bf16 2x2x2 stride-2 transposed convolution (the up-sampling step of the U-Net decoder) on the gfx950
// matrix cores: forward and data gradient.  Both are per-voxel channel mixes, i.e. plain GEMMs whose long
// dimension is the voxel index:
//
//   forward   y[2v + t][co] = bias[co] + sum_ci u[t][ci][co] * x[v][ci]          K = Cin,      8 taps t
//   dgrad     dx[v][ci]     = sum_t sum_co u[t][ci][co] * dy[2v + t][co]         K = 8 * Cout
//
// v_mfma_f32_32x32x16_bf16 with the weights as the A operand (rows = output channels of the product) and
// 32 consecutive coarse voxels of one W row as the B operand (columns): NDHWC keeps a voxel's channels
// contiguous, so a B fragment is one 16-byte global load per lane and needs no LDS.  The weight fragments
// of a workgroup's channel block are built once in LDS (forward: transposed on the way in, because the
// product reduces over ci while u is stored [ci][co]; dgrad: already in fragment order) and re-read for
// every 32-voxel segment.  The result lane layout - lane l holds voxel l % 32 and channels
// 8*(i/4) + 4*(l/32) + i%4 - gives 8-byte stores.  Both kernels are bound by HBM traffic, not by the
// matrix cores; a workgroup is persistent and its 8 waves walk over segments independently.
// 2-D variant (geometry flag `flat`): 1x2x2 windows, 4 taps t = (b, c), u[4][cin][cout]; the fine voxel of
// tap t lies in the coarse voxel's own slice.
#include "common.h"

namespace sp3d {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kT = 512;          // 8 waves, 2 per SIMD
constexpr int C = 32;            // channel block = MFMA rows
constexpr int SEG = 32;          // voxels per segment = MFMA columns
constexpr int kMaxFragKB = 128;  // LDS spent on weight fragments (1 KB each)
constexpr int kGroups = 256;     // workgroups per launch: one per CU

struct UpArgs {
    const uint16_t *in;      // forward: x (coarse);  dgrad: dy (fine)
    const uint16_t *u;       // [8][cin][cout]
    const float *bias;       // forward only, may be null
    uint16_t *out;           // forward: y (fine);  dgrad: dx (coarse)
    Geo gf, gc;
    int cin, cout;
    int nblk;                // channel blocks of the output handled by different workgroups
    int wpb;                 // workgroups per channel block
    int nseg;                // segments per coarse W row
    int nitems;              // segments in total
    int ntap;                // window positions: 8, or 4 in the 2-D variant
};

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    union { bf16x2 v; uint32_t u; } r;
    r.v = __builtin_convertvector(f32x2{a, b}, bf16x2);
    return r.u;
}

// Workgroup ids go round the 8 XCDs; renumbered, an XCD holds a run of neighbouring ids: workgroups that walk
// neighbouring segments, or the channel blocks of the same segments, and share rows and cache lines through the
// XCD's L2.
__device__ __forceinline__ int xcd_block() {
    return (gridDim.x & 7) == 0 ? (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
}

struct Item { int tile, d, h, w0; };
__device__ __forceinline__ Item decode_item(int item, int nseg, const Geo &gc) {
    Item o;
    o.w0 = (item % nseg) * SEG;
    int t = item / nseg;
    o.h = t % gc.th; t /= gc.th;
    o.d = t % gc.td;
    o.tile = t / gc.td;
    return o;
}
// padded voxel index of interior voxel (d, h, w) of a tile
__device__ __forceinline__ size_t pvox(const Geo &g, int tile, int d, int h, int w) {
    return static_cast<size_t>(tile) * g.tile_vox + (static_cast<size_t>(d + 1) * g.ph + h + 1) * g.pw + w + 1;
}

// padded voxel index of the fine voxel that tap t of coarse voxel (d, h, w) produces
__device__ __forceinline__ size_t fvox(const Geo &gf, int tile, int d, int h, int w, int tap) {
    return pvox(gf, tile, gf.flat ? d : 2 * d + (tap >> 2), 2 * h + ((tap >> 1) & 1), 2 * w + (tap & 1));
}

// ---- forward -----------------------------------------------------------------------------------------
// NKS = Cin / 16 reduction steps.  LDS: fragment (tap, ks) at (tap * NKS + ks) KB; lane l of it holds
// u[tap][16 ks + 8 (l/32) + j][32 cb + l % 32], j = 0..7.
template <int NKS>
__global__ __launch_bounds__(kT) void upconv_fwd_mfma_kernel(UpArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int bid = xcd_block();
    const int cb = bid % a.nblk, sub = bid / a.nblk;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int CIN = 16 * NKS;
    // weights: 16-byte pieces (8 output channels of one (tap, ci)) scattered to the 8 lanes that own them
    for (int e = tid; e < a.ntap * CIN * 4; e += kT) {
        const int c8 = e & 3, ci = (e >> 2) % CIN, tap = (e >> 2) / CIN;
        const uint4 v = *reinterpret_cast<const uint4 *>(a.u + (static_cast<size_t>(tap) * CIN + ci) * a.cout +
                                                         C * cb + 8 * c8);
        char *dst = lds + (tap * NKS + (ci >> 4)) * 1024 + ((ci >> 3) & 1) * 512 + (ci & 7) * 2 + 8 * c8 * 16;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 8; ++j)
            *reinterpret_cast<uint16_t *>(dst + j * 16) = static_cast<uint16_t>(w[j >> 1] >> (16 * (j & 1)));
    }
    __syncthreads();

    const int m = lane & 31, kh = lane >> 5;
    float bv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) bv[i] = a.bias ? a.bias[C * cb + 8 * (i >> 2) + 4 * kh + (i & 3)] : 0.f;

    // Items are taken two at a time so that the x fragments of the next one are in flight while the current
    // one is multiplied (the named buffers b0 / b1 swap roles without register copies).
    const int stride = a.wpb * (kT / 64);
    bf16x8 b0[NKS], b1[NKS];
    auto fetch = [&](int item, bf16x8 (&b)[NKS]) {
        if (item >= a.nitems) return;
        const Item o = decode_item(item, a.nseg, a.gc);
        const int w = min(o.w0 + m, a.gc.tw - 1);
        const uint16_t *px = a.in + pvox(a.gc, o.tile, o.d, o.h, w) * CIN + 8 * kh;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) b[ks] = *reinterpret_cast<const bf16x8 *>(px + 16 * ks);
    };
    // Stores.  A lane of D holds 4 x 8 bytes of ONE fine voxel, and neighbouring lanes hold voxels two apart, so
    // direct stores are 8-byte pieces scattered over 4 KB.  With room in LDS (Cin <= 128) the two taps that
    // interleave along W are put together in a wave-private buffer first (64 fine voxels x 64 bytes, rows padded
    // to 72 bytes) and written out as 16-byte pieces that are contiguous across the wave: 1 KB per instruction.
    constexpr bool TR = NKS <= 8;
    constexpr int TROW = 72;
    char *tbuf = lds + 8 * NKS * 1024 + wave * (64 * TROW);
    const int rv = lane >> 2, rp = lane & 3;
    auto compute = [&](int item, const bf16x8 (&b)[NKS]) {
        const Item o = decode_item(item, a.nseg, a.gc);
        const int w = o.w0 + m;
        const bool ok = w < a.gc.tw;
#pragma unroll 1
        for (int tap = 0; tap < a.ntap; ++tap) {
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = bv[i];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const bf16x8 af = *reinterpret_cast<const bf16x8 *>(lds + (tap * NKS + ks) * 1024 + lane * 16);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b[ks], acc, 0, 0, 0);
            }
            if (TR) {
                char *wr = tbuf + (2 * m + (tap & 1)) * TROW + 8 * kh;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2 *>(wr + 16 * q) = make_uint2(pack2(acc[4 * q], acc[4 * q + 1]),
                                                                         pack2(acc[4 * q + 2], acc[4 * q + 3]));
                if (tap & 1) {
                    // both taps of this fine row are in the buffer (the LDS unit serves a wave's accesses in order)
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    uint16_t *prow = a.out + fvox(a.gf, o.tile, o.d, o.h, o.w0, tap & ~1) * a.cout + C * cb + 8 * rp;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int fv = 16 * j + rv;                     // fine voxel of the 64
                        const uint2 lo = *reinterpret_cast<const uint2 *>(tbuf + fv * TROW + 16 * rp);
                        const uint2 hi = *reinterpret_cast<const uint2 *>(tbuf + fv * TROW + 16 * rp + 8);
                        if (2 * o.w0 + fv < 2 * a.gc.tw)
                            st_stream16(prow + static_cast<size_t>(fv) * a.cout, make_uint4(lo.x, lo.y, hi.x, hi.y));
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                }
            } else if (ok) {
                uint16_t *py = a.out + fvox(a.gf, o.tile, o.d, o.h, w, tap) * a.cout + C * cb + 4 * kh;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2 *>(py + 8 * q) = make_uint2(pack2(acc[4 * q], acc[4 * q + 1]),
                                                                       pack2(acc[4 * q + 2], acc[4 * q + 3]));
            }
        }
    };
    int item = sub * (kT / 64) + wave;
    fetch(item, b0);
#pragma unroll 1
    for (; item < a.nitems; item += 2 * stride) {
        fetch(item + stride, b1);
        compute(item, b0);
        if (item + stride >= a.nitems) break;
        fetch(item + 2 * stride, b0);
        compute(item + stride, b1);
    }
}

// ---- data gradient -------------------------------------------------------------------------------------
// NKS = Cout / 16 reduction steps per tap, GCI input-channel blocks per workgroup (they share the dy
// fragments).  LDS: fragment (g, tap, ks) at ((g * 8 + tap) * NKS + ks) KB; lane l holds
// u[tap][32 (cg GCI + g) + l % 32][16 ks + 8 (l/32) + j] - 16 contiguous bytes of u.
template <int NKS, int GCI>
__global__ __launch_bounds__(kT) void upconv_dgrad_mfma_kernel(UpArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int bid = xcd_block();
    const int cg = bid % a.nblk, sub = bid / a.nblk;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int COUT = 16 * NKS;
    const int m = lane & 31, kh = lane >> 5;
    for (int e = tid; e < GCI * 8 * NKS * 64; e += kT) {
        const int l = e & 63, f = e >> 6;
        const int ks = f % NKS, tap = (f / NKS) & 7, g = f / (8 * NKS);
        if (tap >= a.ntap) continue;
        const int ci = C * (cg * GCI + g) + (l & 31);
        *reinterpret_cast<uint4 *>(lds + e * 16) = *reinterpret_cast<const uint4 *>(
            a.u + (static_cast<size_t>(tap) * a.cin + ci) * COUT + 16 * ks + 8 * (l >> 5));
    }
    __syncthreads();

#pragma unroll 1
    for (int item = sub * (kT / 64) + wave; item < a.nitems; item += a.wpb * (kT / 64)) {
        const Item o = decode_item(item, a.nseg, a.gc);
        const int w = o.w0 + m;
        const bool ok = w < a.gc.tw;
        const int wl = ok ? w : a.gc.tw - 1;
        f32x16 acc[GCI];
#pragma unroll
        for (int g = 0; g < GCI; ++g)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[g][i] = 0.f;
        // taps in pairs: the dy fragments of the next tap are in flight while the current one is multiplied
        bf16x8 b0[NKS], b1[NKS];
        auto fetch = [&](int tap, bf16x8 (&b)[NKS]) {
            const uint16_t *pdy = a.in + fvox(a.gf, o.tile, o.d, o.h, wl, tap) * COUT + 8 * kh;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) b[ks] = *reinterpret_cast<const bf16x8 *>(pdy + 16 * ks);
        };
        auto compute = [&](int tap, const bf16x8 (&b)[NKS]) {
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                for (int g = 0; g < GCI; ++g) {
                    const bf16x8 af = *reinterpret_cast<const bf16x8 *>(
                        lds + ((g * 8 + tap) * NKS + ks) * 1024 + lane * 16);
                    acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b[ks], acc[g], 0, 0, 0);
                }
        };
        fetch(0, b0);
#pragma unroll 1
        for (int tap = 0; tap < a.ntap; tap += 2) {
            fetch(tap + 1, b1);
            compute(tap, b0);
            if (tap + 2 < a.ntap) fetch(tap + 2, b0);
            compute(tap + 1, b1);
        }
        if (ok) {
            uint16_t *px = a.out + pvox(a.gc, o.tile, o.d, o.h, w) * a.cin + C * cg * GCI + 4 * kh;
#pragma unroll
            for (int g = 0; g < GCI; ++g)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2 *>(px + C * g + 8 * q) =
                        make_uint2(pack2(acc[g][4 * q], acc[g][4 * q + 1]), pack2(acc[g][4 * q + 2], acc[g][4 * q + 3]));
        }
    }
}

// ---- weight gradient -----------------------------------------------------------------------------------
//   du[t][ci][co] = sum_v x[v][ci] * dy[2v + t][co],   db[co] = sum over fine voxels of dy[.][co]
// The reduction runs over voxels while memory keeps channels contiguous, so both operands go through LDS
// and are read back with the transposing load (4 voxels of one channel per lane and read).  Wave t of a
// workgroup owns tap t.  For every 32-voxel segment the workgroup stages the x rows (NCI blocks of 32 input
// channels) ONCE - every tap multiplies the same ones - and each wave the dy rows of its tap (one block of 32
// output channels), with direct-to-LDS loads into a ring of segments shared by the workgroup, one barrier per
// segment.  (With a private ring per wave, each holding its own copy of the x rows, 144 KB of LDS held two
// segments ahead, 40 % of whose bytes were distinct: the kernel ran at what that much data in flight gives,
// 2.7 - 3.3 TB/s at 512^3 and less below.)  LDS records are voxel-major, 64 bytes (32 channels) per voxel.
// Each workgroup writes its partial sums; a second kernel adds them in workgroup order.
constexpr int wg_ring_slots(int nci) { return nci == 2 ? 7 : 8; }      // 7 x 20 KB, 8 x 18 KB
constexpr int wg_slot_bytes(int nci) { return (nci + 8) * 2048; }      // x blocks, then the dy blocks of the 8 taps

struct UpWArgs {
    const uint16_t *x, *dy;
    float *part_w;           // [workgroup][8][32 NCI][32]
    float *part_b;           // [workgroup][8][32]
    Geo gf, gc;
    int cin, cout;
    int nco;                 // output-channel blocks; channel group = (ci group) * nco + co block
    int ngroups, wpg;        // channel groups, workgroups per group
    int nseg, nitems;
    int ntap;                // window positions: 8, or 4 in the 2-D variant (waves 4..7 then have no tap)
};

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes per lane from global memory to LDS address dst + 16 * lane (dst wave-uniform, in M0).  The wait
// on lgkmcnt makes sure that this wave's earlier reads of the ring slot have returned before it is refilled.
__device__ __forceinline__ void dma16_after_reads(const uint16_t *src, const char *dst) {
    const uint32_t l = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (const __attribute__((address_space(3))) char *)dst));
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(src), "s"(l)
                 : "memory");
}

// One 32x32x16 operand (32 channels x 16 voxels) from 16 voxel records at p (p includes the lane part).
// Lane l gets channel l % 32 and voxels 8 (l/32) + {0..7}; `nvalid` voxels of the 16 are real, the others
// are forced to zero (FULL: all are real).
template <bool FULL>
__device__ __forceinline__ bf16x8 tr_frag(const char *p, int lane, int nvalid) {
    union { struct { s16x4 lo, hi; } s; u32x4 w; bf16x8 v; } u;
    u.s.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(__attribute__((address_space(3))) char *)(p));
    u.s.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(__attribute__((address_space(3))) char *)(p + 4 * 64));
    if (!FULL) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int c = nvalid - (8 * (lane >> 5) + 4 * r);        // real voxels among this read's four
            u.w[2 * r] &= c >= 2 ? 0xffffffffu : (c == 1 ? 0x0000ffffu : 0u);
            u.w[2 * r + 1] &= c >= 4 ? 0xffffffffu : (c == 3 ? 0x0000ffffu : 0u);
        }
    }
    return u.v;
}

template <int NCI, bool FULL>
__global__ __launch_bounds__(kT) void upconv_wgrad_mfma_kernel(UpWArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int SLOT = wg_slot_bytes(NCI), R = wg_ring_slots(NCI);
    constexpr int DM = 3;                            // staging loads per segment and wave
    // neighbours on an XCD (see xcd_block) are the channel groups of ONE share of the items: they walk the same
    // segments together, and the x rows that cout / 32 of them stage, the dy rows that cin / (32 NCI) of them
    // stage, come from the XCD's L2 after the first
    const int bid = xcd_block();
    const int group = bid % a.ngroups, sub = bid / a.ngroups;
    const int cg = group / a.nco, cb = group % a.nco;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // 2-D variant: waves 4 .. 7 have no tap; they stage (their share of x, and the last tap's dy once more) and
    // keep the barriers, nothing else
    const bool active = wave < a.ntap;
    const int tap = active ? wave : a.ntap - 1;
    // transposing-read address of this lane inside a 16-voxel group of records
    const int p16 = lane & 15;
    const int tr_off = (8 * (lane >> 5) + (p16 >> 2)) * 64 + (16 * ((lane >> 4) & 1) + 4 * (p16 & 3)) * 2;
    const int sv = lane >> 2, sc = lane & 3;         // staging: voxel within a 16-voxel group, 16-byte chunk
    // this wave's share of the x rows: one of their 2 NCI loads of 16 voxels (four waves share each when NCI = 1,
    // two when NCI = 2: the same bytes to the same place)
    const int xb = NCI == 2 ? (wave >> 1) & 1 : 0, xq = wave & 1;

    f32x16 acc[NCI], accb;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        accb[i] = 0.f;
#pragma unroll
        for (int b = 0; b < NCI; ++b) acc[b][i] = 0.f;
    }
    union { uint32_t w[4]; bf16x8 v; } ones;
#pragma unroll
    for (int i = 0; i < 4; ++i) ones.w[i] = 0x3f803f80u;
    const bool bias_group = cg == 0;

    auto stage = [&](int item, int slot) {
        const Item o = decode_item(item, a.nseg, a.gc);
        char *dst = lds + slot * SLOT;
        {
            const int w = min(o.w0 + 16 * xq + sv, a.gc.tw - 1);
            const uint16_t *px = a.x + pvox(a.gc, o.tile, o.d, o.h, w) * a.cin + C * cg * NCI + 8 * sc;
            dma16_after_reads(px + C * xb, dst + xb * 2048 + xq * 1024);
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int w = min(o.w0 + 16 * q + sv, a.gc.tw - 1);
            const uint16_t *pz = a.dy + fvox(a.gf, o.tile, o.d, o.h, w, tap) * a.cout + C * cb + 8 * sc;
            dma16_after_reads(pz, dst + (NCI + tap) * 2048 + q * 1024);
        }
    };

    // items sub, sub + wpg, ...  The ring is filled R - 1 segments ahead; past the end the last item is staged
    // again (into slots that are never read), so that every wave always has the same number of loads in flight.
    // Every wave of the workgroup walks the same items, so the barriers match.
    const int first = sub, last = first + ((a.nitems - 1 - first) / a.wpg) * a.wpg;
#pragma unroll
    for (int j = 0; j < R - 1; ++j) stage(min(first + j * a.wpg, last), j);
    int slot = 0;
#pragma unroll 1
    for (int item = first; item <= last; item += a.wpg) {
        // this wave's loads of the item have landed; behind the barrier everybody's have, and every wave has
        // left the item before, whose slot takes the loads of the item R - 1 ahead
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((R - 2) * DM) : "memory");
        __builtin_amdgcn_s_barrier();
        const int nxt = item + (R - 1) * a.wpg;
        stage(nxt <= last ? nxt : last, slot == 0 ? R - 1 : slot - 1);
        if (active) {
            const char *st = lds + slot * SLOT + tr_off;
            const int nvalid = FULL ? 32 : a.gc.tw - (item % a.nseg) * SEG;    // real voxels of the segment
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const bf16x8 zf = tr_frag<FULL>(st + (NCI + tap) * 2048 + ks * 1024, lane, nvalid - 16 * ks);
#pragma unroll
                for (int b = 0; b < NCI; ++b) {
                    const bf16x8 xf = tr_frag<FULL>(st + b * 2048 + ks * 1024, lane, nvalid - 16 * ks);
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, zf, acc[b], 0, 0, 0);
                }
                if (bias_group) accb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones.v, zf, accb, 0, 0, 0);
            }
        }
        slot = slot == R - 1 ? 0 : slot + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (!active) return;

    // lane l holds column co = l % 32 and rows ci = 8 (i/4) + 4 (l/32) + i % 4
    const int wg = group * a.wpg + sub;
    float *pw = a.part_w + (static_cast<size_t>(wg) * 8 + tap) * (NCI * C * C);
#pragma unroll
    for (int b = 0; b < NCI; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            pw[(C * b + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3)) * C + (lane & 31)] = acc[b][i];
    // every row of the ones-product is the column sum; row 0 sits in register 0 of lanes 0..31
    if (lane < C) a.part_b[(static_cast<size_t>(wg) * 8 + tap) * C + lane] = accb[0];
}

// du[t][ci][co] = sum over the workgroups of (ci, co)'s channel group, in workgroup order; db[co] likewise
// over the workgroups of ci group 0 and the 8 taps.
__global__ __launch_bounds__(256) void upconv_wgrad_reduce_kernel(const float *__restrict__ part_w,
                                                                  const float *__restrict__ part_b,
                                                                  float *__restrict__ du, float *__restrict__ db,
                                                                  int cin, int cout, int nci, int wpg, int ntap) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    const int nw = ntap * cin * cout;
    const int nco = cout / C, gci = C * nci;
    if (e < nw) {
        const int co = e % cout, ci = (e / cout) % cin, tap = e / (cout * cin);
        const int group = (ci / gci) * nco + co / C;
        const float *p = part_w + ((static_cast<size_t>(group) * wpg * 8 + tap) * gci + ci % gci) * C + co % C;
        // sixteen loads in flight, added in workgroup order (a chain of dependent loads pays the memory latency
        // once per partial)
        const size_t kstride = static_cast<size_t>(8) * gci * C;
        float s = 0.f;
        int k = 0;
        for (; k + 16 <= wpg; k += 16) {
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) v[i] = p[(k + i) * kstride];
#pragma unroll
            for (int i = 0; i < 16; ++i) s += v[i];
        }
        for (; k < wpg; ++k) s += p[k * kstride];
        du[e] = s;
    } else if (db && e < nw + cout) {
        const int co = e - nw;
        const float *p = part_b + static_cast<size_t>(co / C) * wpg * 8 * C + co % C;      // ci group 0
        float s = 0.f;
        for (int k = 0; k < wpg; ++k)
            for (int t = 0; t < ntap; ++t) s += p[(k * 8 + t) * C];
        db[co] = s;
    }
}

int wgrad_plan(const Geo &gc, int cin, int cout, UpWArgs *a, int *nci) {
    *nci = cin % (2 * C) == 0 ? 2 : 1;
    a->cin = cin; a->cout = cout;
    a->nco = cout / C;
    a->ngroups = (cin / (C * *nci)) * a->nco;
    a->nseg = (gc.tw + SEG - 1) / SEG;
    const long long items = 1LL * gc.ntiles * gc.td * gc.th * a->nseg;
    if (items > 0x7fff0000LL) return SP_EGEOM;
    a->nitems = static_cast<int>(items);
    int wpg = kGroups / a->ngroups;
    if (wpg < 1) wpg = 1;
    if (wpg > items) wpg = static_cast<int>(items);
    a->wpg = wpg;
    return SP_OK;
}

// ---- wide layers (more than 256 channels on the reduction side) -----------------------------------------
// The bottom of a deep U-Net has few voxels and many channels: the weight fragments of all 8 taps no longer
// fit LDS, and the tensors are small enough to be re-read from L2.  Forward: a workgroup serves ONE tap of
// one output block (its fragments: Cin / 16 KB <= 64 KB) and walks over the segments with a single
// accumulator, fetching the x fragments 8 reduction steps at a time.  Data gradient: the weight fragments
// are contiguous 16-byte pieces of u, so they are read straight from global memory (L2) next to the dy
// fragments.
template <int UNUSED = 0>
__global__ __launch_bounds__(kT) void upconv_fwd_mfma_big_kernel(UpArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int bid = xcd_block();
    const int blk = bid % a.nblk, sub = bid / a.nblk;
    const int tap = blk % a.ntap, cb = blk / a.ntap;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nks = a.cin >> 4;
    for (int e = tid; e < a.cin * 4; e += kT) {
        const int c8 = e & 3, ci = e >> 2;
        const uint4 v = *reinterpret_cast<const uint4 *>(a.u + (static_cast<size_t>(tap) * a.cin + ci) * a.cout +
                                                         C * cb + 8 * c8);
        char *dst = lds + (ci >> 4) * 1024 + ((ci >> 3) & 1) * 512 + (ci & 7) * 2 + 8 * c8 * 16;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 8; ++j)
            *reinterpret_cast<uint16_t *>(dst + j * 16) = static_cast<uint16_t>(w[j >> 1] >> (16 * (j & 1)));
    }
    __syncthreads();
    const int m = lane & 31, kh = lane >> 5;
    float bv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) bv[i] = a.bias ? a.bias[C * cb + 8 * (i >> 2) + 4 * kh + (i & 3)] : 0.f;
#pragma unroll 1
    for (int item = sub * (kT / 64) + wave; item < a.nitems; item += a.wpb * (kT / 64)) {
        const Item o = decode_item(item, a.nseg, a.gc);
        const int w = o.w0 + m;
        const bool ok = w < a.gc.tw;
        const uint16_t *px = a.in + pvox(a.gc, o.tile, o.d, o.h, ok ? w : a.gc.tw - 1) * a.cin + 8 * kh;
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = bv[i];
#pragma unroll 1
        for (int k0 = 0; k0 < nks; k0 += 8) {          // nks is a multiple of 2; the chunk may be short
            bf16x8 b[8];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (k0 + k < nks) b[k] = *reinterpret_cast<const bf16x8 *>(px + 16 * (k0 + k));
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (k0 + k < nks) {
                    const bf16x8 af = *reinterpret_cast<const bf16x8 *>(lds + (k0 + k) * 1024 + lane * 16);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b[k], acc, 0, 0, 0);
                }
        }
        if (ok) {
            uint16_t *py = a.out + fvox(a.gf, o.tile, o.d, o.h, w, tap) * a.cout + C * cb + 4 * kh;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<uint2 *>(py + 8 * q) = make_uint2(pack2(acc[4 * q], acc[4 * q + 1]),
                                                                   pack2(acc[4 * q + 2], acc[4 * q + 3]));
        }
    }
}

template <int UNUSED = 0>
__global__ __launch_bounds__(kT) void upconv_dgrad_mfma_big_kernel(UpArgs a) {
    const int bid = xcd_block();
    const int cg = bid % a.nblk, sub = bid / a.nblk;      // one input-channel block per workgroup
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nks = a.cout >> 4;
    const int m = lane & 31, kh = lane >> 5;
    // this lane's row of u: input channel 32 cg + lane % 32, reduction offset 8 (lane / 32)
    const uint16_t *urow = a.u + static_cast<size_t>(C * cg + m) * a.cout + 8 * kh;
    const size_t utap = static_cast<size_t>(a.cin) * a.cout;
#pragma unroll 1
    for (int item = sub * (kT / 64) + wave; item < a.nitems; item += a.wpb * (kT / 64)) {
        const Item o = decode_item(item, a.nseg, a.gc);
        const int w = o.w0 + m;
        const bool ok = w < a.gc.tw;
        const int wl = ok ? w : a.gc.tw - 1;
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll 1
        for (int tap = 0; tap < a.ntap; ++tap) {
            const uint16_t *pdy = a.in + fvox(a.gf, o.tile, o.d, o.h, wl, tap) * a.cout + 8 * kh;
            const uint16_t *pu = urow + tap * utap;
#pragma unroll 1
            for (int k0 = 0; k0 < nks; k0 += 8) {
                bf16x8 b[8], af[8];
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (k0 + k < nks) {
                        b[k] = *reinterpret_cast<const bf16x8 *>(pdy + 16 * (k0 + k));
                        af[k] = *reinterpret_cast<const bf16x8 *>(pu + 16 * (k0 + k));
                    }
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (k0 + k < nks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[k], b[k], acc, 0, 0, 0);
            }
        }
        if (ok) {
            uint16_t *px = a.out + pvox(a.gc, o.tile, o.d, o.h, w) * a.cin + C * cg + 4 * kh;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<uint2 *>(px + 8 * q) = make_uint2(pack2(acc[4 * q], acc[4 * q + 1]),
                                                                   pack2(acc[4 * q + 2], acc[4 * q + 3]));
        }
    }
}

int dgrad_gci(int cin, int cout) {
    int g = 4;
    while (g > 1 && (g * 8 * (cout / 16) > kMaxFragKB || (cin / C) % g != 0)) g >>= 1;
    return g;
}

int plan(const Geo &gc, int nblk, UpArgs *a) {
    a->nblk = nblk;
    a->nseg = (gc.tw + SEG - 1) / SEG;
    const long long items = 1LL * gc.ntiles * gc.td * gc.th * a->nseg;
    if (items > 0x7fff0000LL) return SP_EGEOM;
    a->nitems = static_cast<int>(items);
    int wpb = kGroups / nblk;
    if (wpb < 1) wpb = 1;
    const long long need = (items + kT / 64 - 1) / (kT / 64);      // workgroups that would each get one pass
    if (wpb > need) wpb = static_cast<int>(need);
    a->wpb = wpb;
    return SP_OK;
}

template <typename K>
int launch(K kernel, const UpArgs &a, int lds_bytes, hipStream_t s) {
    // more than 64 KB of dynamic LDS has to be requested explicitly (cheap; repeated per launch so that
    // every instantiation is covered)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return record_hip(e);
    hipLaunchKernelGGL(kernel, dim3(a.nblk * a.wpb), dim3(kT), lds_bytes, s, a);
    return record_hip(hipGetLastError());
}

}  // namespace

bool upconv_mfma_supported(const Geo &gf, const Geo &gc, int cin, int cout, sp_dtype_t dt) {
    if (dt != SP_BF16 || cin % C != 0 || cout % C != 0 || cin > 1024 || cout > 1024) return false;
    // element offsets of a voxel inside the tensors stay far below 2^63; segment counts are checked in plan()
    return 1LL * gc.ntiles * gc.td * gc.th * ((gc.tw + SEG - 1) / SEG) <= 0x7fff0000LL;
}

int launch_upconv_fwd_mfma(const void *Px, const void *u, const float *bias, void *Py, const Geo &gf, const Geo &gc,
                           int cin, int cout, hipStream_t s) {
    UpArgs a;
    a.in = static_cast<const uint16_t *>(Px);
    a.u = static_cast<const uint16_t *>(u);
    a.bias = bias;
    a.out = static_cast<uint16_t *>(Py);
    a.gf = gf; a.gc = gc; a.cin = cin; a.cout = cout;
    a.ntap = gf.flat ? 4 : 8;
    if (cin > 256) {                 // one tap per workgroup: ntap x (cout / 32) kinds of workgroups
        int rc = plan(gc, a.ntap * (cout / C), &a);
        if (rc != SP_OK) return rc;
        return launch(upconv_fwd_mfma_big_kernel<0>, a, (cin / 16) * 1024, s);
    }
    int rc = plan(gc, cout / C, &a);
    if (rc != SP_OK) return rc;
    // weight fragments, plus (Cin <= 128) one 64-voxel store buffer per wave
    const int lds_bytes = 8 * (cin / 16) * 1024 + (cin <= 128 ? (kT / 64) * 64 * 72 : 0);
    switch (cin / C) {
    case 1: return launch(upconv_fwd_mfma_kernel<2>, a, lds_bytes, s);
    case 2: return launch(upconv_fwd_mfma_kernel<4>, a, lds_bytes, s);
    case 3: return launch(upconv_fwd_mfma_kernel<6>, a, lds_bytes, s);
    case 4: return launch(upconv_fwd_mfma_kernel<8>, a, lds_bytes, s);
    case 5: return launch(upconv_fwd_mfma_kernel<10>, a, lds_bytes, s);
    case 6: return launch(upconv_fwd_mfma_kernel<12>, a, lds_bytes, s);
    case 7: return launch(upconv_fwd_mfma_kernel<14>, a, lds_bytes, s);
    case 8: return launch(upconv_fwd_mfma_kernel<16>, a, lds_bytes, s);
    default: return SP_EUNSUPPORTED;
    }
}

int launch_upconv_dgrad_mfma(const void *Pdy, const void *u, void *Pdx, const Geo &gf, const Geo &gc, int cin,
                             int cout, hipStream_t s) {
    UpArgs a;
    a.in = static_cast<const uint16_t *>(Pdy);
    a.u = static_cast<const uint16_t *>(u);
    a.bias = nullptr;
    a.out = static_cast<uint16_t *>(Pdx);
    a.gf = gf; a.gc = gc; a.cin = cin; a.cout = cout;
    a.ntap = gf.flat ? 4 : 8;
    if (cout > 256) {                // weight fragments straight from global memory
        int rc = plan(gc, cin / C, &a);
        if (rc != SP_OK) return rc;
        hipLaunchKernelGGL(upconv_dgrad_mfma_big_kernel<0>, dim3(a.nblk * a.wpb), dim3(kT), 0, s, a);
        return record_hip(hipGetLastError());
    }
    const int gci = dgrad_gci(cin, cout);
    int rc = plan(gc, cin / C / gci, &a);
    if (rc != SP_OK) return rc;
    const int nks = cout / 16;
    const int lds_bytes = gci * 8 * nks * 1024;
#define SP3D_DG(NKS)                                                                       \
    case NKS:                                                                              \
        if (gci == 4) return launch(upconv_dgrad_mfma_kernel<NKS, 4>, a, lds_bytes, s);    \
        if (gci == 2) return launch(upconv_dgrad_mfma_kernel<NKS, 2>, a, lds_bytes, s);    \
        return launch(upconv_dgrad_mfma_kernel<NKS, 1>, a, lds_bytes, s);
    switch (nks) {
        SP3D_DG(2) SP3D_DG(4) SP3D_DG(6) SP3D_DG(8) SP3D_DG(10) SP3D_DG(12) SP3D_DG(14) SP3D_DG(16)
    default: return SP_EUNSUPPORTED;
    }
#undef SP3D_DG
}

size_t upconv_wgrad_mfma_ws_bytes(const Geo &gc, int cin, int cout) {
    UpWArgs a;
    int nci;
    if (wgrad_plan(gc, cin, cout, &a, &nci) != SP_OK) return 0;
    return static_cast<size_t>(a.ngroups) * a.wpg * 8 * (nci * C * C + C) * sizeof(float);
}

int launch_upconv_wgrad_mfma(const void *Px, const void *Pdy, float *du, float *db, const Geo &gf, const Geo &gc,
                             int cin, int cout, void *ws, hipStream_t s) {
    UpWArgs a;
    int nci;
    int rc = wgrad_plan(gc, cin, cout, &a, &nci);
    if (rc != SP_OK) return rc;
    a.x = static_cast<const uint16_t *>(Px);
    a.dy = static_cast<const uint16_t *>(Pdy);
    a.gf = gf; a.gc = gc;
    a.ntap = gf.flat ? 4 : 8;
    a.part_w = static_cast<float *>(ws);
    a.part_b = a.part_w + static_cast<size_t>(a.ngroups) * a.wpg * 8 * nci * C * C;
    const bool full = gc.tw % SEG == 0;
    const int lds_bytes = wg_ring_slots(nci) * wg_slot_bytes(nci);
    hipError_t e = hipSuccess;
    const dim3 grid(a.ngroups * a.wpg), block(kT);
#define SP3D_UW(NCI, FULL)                                                                              \
    do {                                                                                                \
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(upconv_wgrad_mfma_kernel<NCI, FULL>),    \
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);                 \
        if (e == hipSuccess)                                                                            \
            hipLaunchKernelGGL((upconv_wgrad_mfma_kernel<NCI, FULL>), grid, block, lds_bytes, s, a);    \
    } while (0)
    if (nci == 2) { if (full) SP3D_UW(2, true); else SP3D_UW(2, false); }
    else { if (full) SP3D_UW(1, true); else SP3D_UW(1, false); }
#undef SP3D_UW
    if (e != hipSuccess) return record_hip(e);
    rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    const int n = a.ntap * cin * cout + cout;
    hipLaunchKernelGGL(upconv_wgrad_reduce_kernel, dim3((n + 255) / 256), dim3(256), 0, s, a.part_w, a.part_b, du,
                       db, cin, cout, nci, a.wpg, a.ntap);
    return record_hip(hipGetLastError());
}

}  // namespace sp3d
