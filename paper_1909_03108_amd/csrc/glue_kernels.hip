// U-Net glue on padded tiles: 2x2x2 max pooling (forward / backward), 2x2x2 stride-2 transposed
// convolution (forward / data gradient / weight gradient), channel concatenation and split.
// Pooling and up-convolution windows never straddle tiles (tile extents are even), so these
// operations need no halo; they read and write tile interiors only.  "Fine" is the higher-resolution
// side (pool input, up-conv output), "coarse" the other; both live on the same tile grid.
// All arithmetic is fp32 (fused multiply-add), inputs f32 or bf16, one rounding on store.
#include "common.h"

namespace sp3d {

namespace {

constexpr int kThreads = 256;

template <typename E> __device__ __forceinline__ float ldf(const E *p, long long i);
template <> __device__ __forceinline__ float ldf<float>(const float *p, long long i) { return p[i]; }
template <> __device__ __forceinline__ float ldf<uint16_t>(const uint16_t *p, long long i) {
    return bf16_to_f32(p[i]);
}
template <typename E> __device__ __forceinline__ void stf(E *p, long long i, float v);
template <> __device__ __forceinline__ void stf<float>(float *p, long long i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void stf<uint16_t>(uint16_t *p, long long i, float v) {
    p[i] = f32_to_bf16(v);
}

// Thread layout shared by the kernels below: a block covers kThreads/cw voxels x cw channel lanes
// (cw = power of two >= min(C, 256)); channels beyond cw are looped over.
struct Lay {
    int cw, cshift;          // channel lanes per voxel and log2
    unsigned nvox;           // voxels to cover (interior voxels of all tiles of the indexing geometry)
    FastDiv int_vox, hw, w;  // decode voxel -> (tile, ld, lh, lw) of the indexing geometry
};

Lay make_lay(const Geo &g, int c) {
    Lay l;
    l.cw = 1; l.cshift = 0;
    while (l.cw < c && l.cw < kThreads) { l.cw <<= 1; ++l.cshift; }
    l.nvox = static_cast<unsigned>(1LL * g.ntiles * g.int_vox);
    l.int_vox = make_fastdiv(static_cast<uint32_t>(g.int_vox));
    l.hw = make_fastdiv(static_cast<uint32_t>(g.th) * g.tw);
    l.w = make_fastdiv(g.tw);
    return l;
}

// two bf16 in a word -> 0xffff in each half whose value is positive (not zero, not negative, not NaN)
__device__ __forceinline__ uint32_t positive_halves(uint32_t v) {
    const uint32_t lo = v & 0xffffu, hi = v >> 16;
    return ((lo - 1u) < 0x7f80u ? 0x0000ffffu : 0u) | ((hi - 1u) < 0x7f80u ? 0xffff0000u : 0u);
}

struct Vox { unsigned tile, ld, lh, lw; };
__device__ __forceinline__ Vox decode(unsigned v, const Lay &l) {
    Vox o;
    o.tile = fdiv(v, l.int_vox);
    const unsigned r = fmod_(v, o.tile, l.int_vox);
    o.ld = fdiv(r, l.hw);
    const unsigned q = fmod_(r, o.ld, l.hw);
    o.lh = fdiv(q, l.w);
    o.lw = fmod_(q, o.lh, l.w);
    return o;
}
// padded voxel index of interior voxel (ld, lh, lw) of a tile (halo = 1)
__device__ __forceinline__ long long pidx(const Geo &g, unsigned tile, unsigned ld, unsigned lh, unsigned lw) {
    return tile * g.tile_vox + (1LL * (ld + 1) * g.ph + lh + 1) * g.pw + lw + 1;
}

// Workgroup ids go round the 8 XCDs of the chip; with block i working on the i-th run of voxels every XCD touches
// every eighth run.  Renumbered (when the grid is a multiple of 8), each XCD streams through one contiguous
// eighth of the voxels: the pooling kernels, which touch 2 x 2 x 2 rows of the fine tensor per row of the coarse
// one, run 5 - 6 % faster that way (the one-voxel-per-thread kernels of the 1x1x1 head 2 - 4 % slower: not used there).
__device__ __forceinline__ unsigned xcd_block() {
    return (gridDim.x & 7u) == 0 ? (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
}

// Fine-tensor position k of the window that belongs to coarse voxel o: 2x2x2 windows, k = 4a + 2b + c for
// offset (a, b, c); in the 2-D variant (g.flat) 1x2x2 windows inside the voxel's own slice, k = 2b + c.
template <int NW>
__device__ __forceinline__ long long wpos(const Geo &gf, const Vox &o, int k) {
    if (NW == 4) return pidx(gf, o.tile, o.ld, 2 * o.lh + ((k >> 1) & 1), 2 * o.lw + (k & 1));
    return pidx(gf, o.tile, 2 * o.ld + (k >> 2), 2 * o.lh + ((k >> 1) & 1), 2 * o.lw + (k & 1));
}
__device__ __forceinline__ long long wpos(const Geo &gf, const Vox &o, int k) {
    return gf.flat ? wpos<4>(gf, o, k) : wpos<8>(gf, o, k);
}

// ---- max pooling -------------------------------------------------------------------------------
// One thread per (coarse voxel, channel).  Forward: y = max of the NW window values (8, or 4 in the 2-D
// variant).  Backward: dx of the FIRST maximum in (d,h,w) scan order receives dy, the others receive 0.
// MODE kPoolBwdJoin: the backward pass of an encoder level in one sweep.  The pooled tensor x is also the
// level's ReLU output that the decoder took as its skip input, so the gradient that reaches the level's last
// convolution is  dz = [x > 0] * (maxpool_bwd(x, dy) + skip_grad);  `skip` may be the same tensor as `out`
// (a thread reads its eight positions before it writes them).  The sum is taken in fp32 and rounded once,
// as sp_add does.
enum PoolMode { kPoolFwd = 0, kPoolBwd = 1, kPoolBwdJoin = 2 };
template <typename E, int MODE, int NW>
__global__ __launch_bounds__(kThreads) void maxpool2_kernel(const E *__restrict__ x, const E *__restrict__ dy,
                                                            const E *skip, E *out, Geo gf, Geo gc, Lay l, int C) {
    const unsigned v = blockIdx.x * (kThreads >> l.cshift) + (threadIdx.x >> l.cshift);
    if (v >= l.nvox) return;
    const Vox o = decode(v, l);
    const long long pc = pidx(gc, o.tile, o.ld, o.lh, o.lw);
    long long pf[NW];
#pragma unroll
    for (int k = 0; k < NW; ++k) pf[k] = wpos<NW>(gf, o, k);
    for (int c = threadIdx.x & (l.cw - 1); c < C; c += l.cw) {
        float xv[NW];
#pragma unroll
        for (int k = 0; k < NW; ++k) xv[k] = ldf<E>(x, pf[k] * C + c);
        float best = xv[0];
        int arg = 0;
#pragma unroll
        for (int k = 1; k < NW; ++k)
            if (xv[k] > best) { best = xv[k]; arg = k; }
        if (MODE == kPoolBwd) {
            const E g = dy[pc * C + c];
#pragma unroll
            for (int k = 0; k < NW; ++k) out[pf[k] * C + c] = k == arg ? g : E(0);
        } else if (MODE == kPoolBwdJoin) {
            const float g = ldf<E>(dy, pc * C + c);
            float sk[NW];
#pragma unroll
            for (int k = 0; k < NW; ++k) sk[k] = ldf<E>(skip, pf[k] * C + c);
#pragma unroll
            for (int k = 0; k < NW; ++k) stf<E>(out, pf[k] * C + c, xv[k] > 0.f ? (k == arg ? g : 0.f) + sk[k] : 0.f);
        } else {
            stf<E>(out, pc * C + c, best);
        }
    }
}

// The same three operations for bf16 tensors whose channel count is a multiple of 8: a thread owns 8 channels
// (16 bytes) of a coarse voxel, so every access is a full 16-byte piece and C / 8 consecutive lanes cover a
// voxel record back to back.  Comparisons and the sum are taken on the widened values exactly as above.
template <int MODE, int NW>
__global__ __launch_bounds__(kThreads) void maxpool2_x8_kernel(const uint16_t *__restrict__ x,
                                                               const uint16_t *__restrict__ dy, const uint16_t *skip,
                                                               uint16_t *out, Geo gf, Geo gc, Lay l, int C) {
    const unsigned v = xcd_block() * (kThreads >> l.cshift) + (threadIdx.x >> l.cshift);
    if (v >= l.nvox) return;
    const Vox o = decode(v, l);
    const long long pc = pidx(gc, o.tile, o.ld, o.lh, o.lw);
    long long pf[NW];
#pragma unroll
    for (int k = 0; k < NW; ++k) pf[k] = wpos<NW>(gf, o, k);
    auto widen8 = [](const uint4 &q, float (&f)[8]) {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    };
    auto narrow8 = [](const float (&f)[8]) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = static_cast<uint32_t>(f32_to_bf16(f[2 * i])) | (static_cast<uint32_t>(f32_to_bf16(f[2 * i + 1])) << 16);
        return make_uint4(w[0], w[1], w[2], w[3]);
    };
    for (int cg = threadIdx.x & (l.cw - 1); 8 * cg < C; cg += l.cw) {
        float xv[NW][8];
#pragma unroll
        for (int k = 0; k < NW; ++k) widen8(*reinterpret_cast<const uint4 *>(x + pf[k] * C + 8 * cg), xv[k]);
        float best[8];
        int arg[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            best[e] = xv[0][e];
            arg[e] = 0;
#pragma unroll
            for (int k = 1; k < NW; ++k)
                if (xv[k][e] > best[e]) { best[e] = xv[k][e]; arg[e] = k; }
        }
        if (MODE == kPoolFwd) {
            st_stream16(out + pc * C + 8 * cg, narrow8(best));
            continue;
        }
        float g[8];
        widen8(*reinterpret_cast<const uint4 *>(dy + pc * C + 8 * cg), g);
        uint4 sk[NW];
        if (MODE == kPoolBwdJoin) {
#pragma unroll
            for (int k = 0; k < NW; ++k) sk[k] = *reinterpret_cast<const uint4 *>(skip + pf[k] * C + 8 * cg);
        }
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            float r[8];
            if (MODE == kPoolBwdJoin) {
                float s8[8];
                widen8(sk[k], s8);
#pragma unroll
                for (int e = 0; e < 8; ++e) r[e] = xv[k][e] > 0.f ? (arg[e] == k ? g[e] : 0.f) + s8[e] : 0.f;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) r[e] = arg[e] == k ? g[e] : 0.f;
            }
            st_stream16(out + pf[k] * C + 8 * cg, narrow8(r));
        }
    }
}

// ---- transposed convolution 2x2x2, stride 2 ----------------------------------------------------------
// Forward: one thread per (fine voxel, co): y = bias + sum_ci x[coarse][ci] * u[a][b][c][ci][co].
template <typename E>
__global__ __launch_bounds__(kThreads) void upconv2_fwd_kernel(const E *__restrict__ x, const E *__restrict__ u,
                                                               const float *__restrict__ bias, E *__restrict__ y,
                                                               Geo gf, Geo gc, Lay l, int cin, int cout) {
    const unsigned v = blockIdx.x * (kThreads >> l.cshift) + (threadIdx.x >> l.cshift);
    if (v >= l.nvox) return;
    const Vox o = decode(v, l);                                     // fine voxel
    const int k = (gf.flat ? 0 : (o.ld & 1) << 2) | ((o.lh & 1) << 1) | (o.lw & 1);
    const E *xin = x + pidx(gc, o.tile, gf.flat ? o.ld : o.ld >> 1, o.lh >> 1, o.lw >> 1) * cin;
    const E *uk = u + 1LL * k * cin * cout;
    const long long po = pidx(gf, o.tile, o.ld, o.lh, o.lw);
    for (int co = threadIdx.x & (l.cw - 1); co < cout; co += l.cw) {
        float acc = bias ? bias[co] : 0.f;
        for (int ci = 0; ci < cin; ++ci) acc = fmaf(ldf<E>(xin, ci), ldf<E>(uk, 1LL * ci * cout + co), acc);
        stf<E>(y, po * cout + co, acc);
    }
}

// Data gradient: one thread per (coarse voxel, ci): dx = sum_{window k, co} dy[fine k][co] * u[k][ci][co].
template <typename E>
__global__ __launch_bounds__(kThreads) void upconv2_dgrad_kernel(const E *__restrict__ dy, const E *__restrict__ u,
                                                                 E *__restrict__ dx, Geo gf, Geo gc, Lay l,
                                                                 int cin, int cout) {
    const unsigned v = blockIdx.x * (kThreads >> l.cshift) + (threadIdx.x >> l.cshift);
    if (v >= l.nvox) return;
    const Vox o = decode(v, l);                                     // coarse voxel
    const long long po = pidx(gc, o.tile, o.ld, o.lh, o.lw);
    for (int ci = threadIdx.x & (l.cw - 1); ci < cin; ci += l.cw) {
        float acc = 0.f;
        for (int k = 0; k < (gf.flat ? 4 : 8); ++k) {
            const E *g = dy + wpos(gf, o, k) * cout;
            const E *uk = u + (1LL * k * cin + ci) * cout;
            for (int co = 0; co < cout; ++co) acc = fmaf(ldf<E>(g, co), ldf<E>(uk, co), acc);
        }
        stf<E>(dx, po * cin + ci, acc);
    }
}

// Data gradient, bf16 with cout a multiple of 8: same thread layout, but dy and the weight row
// u[k][ci][.] are read 8 channels (16 bytes) at a time.
__global__ __launch_bounds__(kThreads) void upconv2_dgrad_bf16x8_kernel(const uint16_t *__restrict__ dy,
                                                                        const uint16_t *__restrict__ u,
                                                                        uint16_t *__restrict__ dx, Geo gf, Geo gc,
                                                                        Lay l, int cin, int cout) {
    const unsigned v = blockIdx.x * (kThreads >> l.cshift) + (threadIdx.x >> l.cshift);
    if (v >= l.nvox) return;
    const Vox o = decode(v, l);                                     // coarse voxel
    const long long po = pidx(gc, o.tile, o.ld, o.lh, o.lw);
    for (int ci = threadIdx.x & (l.cw - 1); ci < cin; ci += l.cw) {
        float acc = 0.f;
        for (int k = 0; k < (gf.flat ? 4 : 8); ++k) {
            const uint4 *g = reinterpret_cast<const uint4 *>(dy + wpos(gf, o, k) * cout);
            const uint4 *uk = reinterpret_cast<const uint4 *>(u + (1LL * k * cin + ci) * cout);
            for (int c8 = 0; c8 < cout / 8; ++c8) {
                const uint4 a = g[c8], b = uk[c8];
                const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc = fmaf(__uint_as_float(aw[e] << 16), __uint_as_float(bw[e] << 16), acc);
                    acc = fmaf(__uint_as_float(aw[e] & 0xffff0000u), __uint_as_float(bw[e] & 0xffff0000u), acc);
                }
            }
        }
        dx[po * cin + ci] = f32_to_bf16(acc);
    }
}

// Weight gradient, stage 1 (same scheme as the direct 3x3x3 weight gradient): block (k*cin + ci, chunk of
// coarse voxels, co group); threads [voxel lane][co]; fixed-order sums; partials to ws[chunk][k][ci][co].
template <typename E>
__global__ __launch_bounds__(kThreads) void upconv2_wgrad_kernel(const E *__restrict__ x, const E *__restrict__ dy,
                                                                 float *__restrict__ part, Geo gf, Geo gc, Lay l,
                                                                 int cin, int cout, int cw, unsigned chunk_vox) {
    __shared__ float red[kThreads];
    const int kci = blockIdx.x, chunk = blockIdx.y;
    const int k = kci / cin, ci = kci % cin;
    const int nvl = kThreads / cw;
    const int col = threadIdx.x % cw, vl = threadIdx.x / cw;
    const int co = blockIdx.z * cw + col;
    float acc = 0.f;
    unsigned v1 = (chunk + 1u) * chunk_vox;
    if (v1 > l.nvox) v1 = l.nvox;
    if (vl < nvl && co < cout) {
        for (unsigned v = chunk * chunk_vox + vl; v < v1; v += nvl) {
            const Vox o = decode(v, l);                             // coarse voxel
            const long long px = pidx(gc, o.tile, o.ld, o.lh, o.lw);
            const long long pz = wpos(gf, o, k);
            acc = fmaf(ldf<E>(x, px * cin + ci), ldf<E>(dy, pz * cout + co), acc);
        }
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (vl == 0 && co < cout) {
        float s = 0.f;
        for (int i = 0; i < nvl; ++i) s += red[i * cw + col];
        part[(1LL * chunk * gridDim.x + kci) * cout + co] = s;
    }
}

// Weight gradient, stage 1, bf16 with cout/8 a power of two <= 256: thread (ci, group of 8 co) keeps the
// 8 window positions x 8 channels of its du entries in registers and walks over the chunk's coarse
// voxels in index order (one 2-byte x load and eight 16-byte dy loads per 64 multiply-adds).
__global__ __launch_bounds__(kThreads) void upconv2_wgrad_bf16x8_kernel(const uint16_t *__restrict__ x,
                                                                        const uint16_t *__restrict__ dy,
                                                                        float *__restrict__ part, Geo gf, Geo gc,
                                                                        Lay l, int cin, int cout, int co8_shift,
                                                                        unsigned chunk_vox) {
    const int co8 = threadIdx.x & ((1 << co8_shift) - 1);
    const int ci = blockIdx.x * (kThreads >> co8_shift) + (threadIdx.x >> co8_shift);
    const int chunk = blockIdx.y;
    if (ci >= cin) return;
    const int nk = gf.flat ? 4 : 8;          // window positions
    float acc[8][8];
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[k][e] = 0.f;
    unsigned v1 = (chunk + 1u) * chunk_vox;
    if (v1 > l.nvox) v1 = l.nvox;
    for (unsigned v = chunk * chunk_vox; v < v1; ++v) {
        const Vox o = decode(v, l);                                 // coarse voxel
        const float xv = bf16_to_f32(x[pidx(gc, o.tile, o.ld, o.lh, o.lw) * cin + ci]);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if (k < nk) {
                const uint4 g = *reinterpret_cast<const uint4 *>(dy + wpos(gf, o, k) * cout + 8 * co8);
                const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[k][2 * e] = fmaf(xv, __uint_as_float(gw[e] << 16), acc[k][2 * e]);
                    acc[k][2 * e + 1] = fmaf(xv, __uint_as_float(gw[e] & 0xffff0000u), acc[k][2 * e + 1]);
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (k < nk) {
            float *p = part + ((1LL * chunk * nk + k) * cin + ci) * cout + 8 * co8;
            *reinterpret_cast<float4 *>(p) = make_float4(acc[k][0], acc[k][1], acc[k][2], acc[k][3]);
            *reinterpret_cast<float4 *>(p + 4) = make_float4(acc[k][4], acc[k][5], acc[k][6], acc[k][7]);
        }
    }
}

// Bias gradient of the up-convolution, stage 1: sum of dy over chunks of FINE interior voxels.
template <typename E>
__global__ __launch_bounds__(kThreads) void bsum_kernel(const E *__restrict__ dy, float *__restrict__ part, Geo g,
                                                        Lay l, int cout, int cw, unsigned chunk_vox) {
    __shared__ float red[kThreads];
    const int chunk = blockIdx.y;
    const int nvl = kThreads / cw;
    const int col = threadIdx.x % cw, vl = threadIdx.x / cw;
    const int co = blockIdx.z * cw + col;
    float acc = 0.f;
    unsigned v1 = (chunk + 1u) * chunk_vox;
    if (v1 > l.nvox) v1 = l.nvox;
    if (vl < nvl && co < cout) {
        for (unsigned v = chunk * chunk_vox + vl; v < v1; v += nvl) {
            const Vox o = decode(v, l);
            acc += ldf<E>(dy, pidx(g, o.tile, o.ld, o.lh, o.lw) * cout + co);
        }
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (vl == 0 && co < cout) {
        float s = 0.f;
        for (int i = 0; i < nvl; ++i) s += red[i * cw + col];
        part[1LL * chunk * cout + co] = s;
    }
}

// ---- channel concat / split: one thread per (padded voxel, channel of the wide tensor) --------------
template <typename E, bool SPLIT>
__global__ __launch_bounds__(kThreads) void concat_kernel(E *__restrict__ a, int ca, E *__restrict__ b, int cb,
                                                          E *__restrict__ c, size_t total) {
    const size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i >= total) return;
    const int cc = ca + cb;
    const size_t v = i / cc;
    const int ch = static_cast<int>(i % cc);
    E *narrow = ch < ca ? a + v * ca + ch : b + v * cb + (ch - ca);
    if (SPLIT) *narrow = c[i]; else c[i] = *narrow;
}

template <typename E>
// (no __restrict__: the output may be the same tensor as either input; every thread reads and writes its own index)
__global__ __launch_bounds__(kThreads) void add_kernel(const E *a, const E *b, E *o, size_t n) {
    const size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i < n) stf<E>(o, i, ldf<E>(a, i) + ldf<E>(b, i));
}

// chunking of the coarse voxels for the up-convolution weight gradient: short chunks (many
// workgroups) as long as the partial sums stay below 256 MB
// concat / split in 16-byte chunks (bf16, both channel counts multiples of 8)
template <bool SPLIT>
__global__ __launch_bounds__(kThreads) void concat_x8_kernel(uint4 *__restrict__ a, int ca8, uint4 *__restrict__ b,
                                                             int cb8, uint4 *__restrict__ c, size_t total) {
    const size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i >= total) return;
    const int cc = ca8 + cb8;
    const size_t v = i / cc;
    const int ch = static_cast<int>(i % cc);
    uint4 *narrow = ch < ca8 ? a + v * ca8 + ch : b + v * cb8 + (ch - ca8);
    if (SPLIT) *narrow = c[i]; else c[i] = *narrow;
}

// element-wise sum, bf16, 8 elements per thread
__global__ __launch_bounds__(kThreads) void add_bf16x8_kernel(const uint4 *a, const uint4 *b, uint4 *o, size_t nvec) {
    const size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i >= nvec) return;
    const uint4 x = a[i], y = b[i];
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
    uint32_t r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float lo = __uint_as_float(xs[k] << 16) + __uint_as_float(ys[k] << 16);
        const float hi = __uint_as_float(xs[k] & 0xffff0000u) + __uint_as_float(ys[k] & 0xffff0000u);
        r[k] = static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
    }
    o[i] = make_uint4(r[0], r[1], r[2], r[3]);
}

// ---- 1x1x1 convolution with a few output channels (the segmentation head), bf16 ----------------------
// These are bound by HBM traffic: every voxel record is read (or written) once with 16-byte accesses,
// the cin x CO weights sit in LDS as floats and are read as broadcasts.  One thread per interior voxel.
constexpr int kPwMaxCin = 256;

template <int CO>
__global__ __launch_bounds__(kThreads) void pointwise_small_fwd_kernel(const uint16_t *__restrict__ x,
                                                                       const uint16_t *__restrict__ p,
                                                                       const float *__restrict__ bias,
                                                                       uint16_t *__restrict__ y, Geo g, Lay l,
                                                                       int cin, int relu) {
    __shared__ float w[kPwMaxCin * CO];
    for (int i = threadIdx.x; i < cin * CO; i += kThreads) w[i] = bf16_to_f32(p[i]);
    __syncthreads();
    const unsigned v = blockIdx.x * kThreads + threadIdx.x;
    if (v >= l.nvox) return;
    const Vox o = decode(v, l);
    const long long pv = pidx(g, o.tile, o.ld, o.lh, o.lw);
    float acc[CO];
#pragma unroll
    for (int co = 0; co < CO; ++co) acc[co] = bias ? bias[co] : 0.f;
    const uint4 *px = reinterpret_cast<const uint4 *>(x + pv * cin);
    for (int c8 = 0; c8 < cin / 8; ++c8) {
        const uint4 q = px[c8];
        const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float xv = __uint_as_float((e & 1) ? (qw[e >> 1] & 0xffff0000u) : (qw[e >> 1] << 16));
#pragma unroll
            for (int co = 0; co < CO; ++co) acc[co] = fmaf(xv, w[(8 * c8 + e) * CO + co], acc[co]);
        }
    }
#pragma unroll
    for (int co = 0; co < CO; ++co) y[pv * CO + co] = f32_to_bf16(relu ? fmaxf(acc[co], 0.f) : acc[co]);
}

// dx[v][ci] = sum_co dy[v][co] * p[ci][co].  cin / 8 consecutive lanes share a voxel, 8 channels (16 bytes) each,
// so that a wave's store (and its mask load) covers whole voxel records back to back.
template <int CO>
__global__ __launch_bounds__(kThreads) void pointwise_small_dgrad_kernel(const uint16_t *__restrict__ dy,
                                                                         const uint16_t *__restrict__ p,
                                                                         uint16_t *__restrict__ dx, Geo g, Lay l,
                                                                         int cin, int cg_shift,
                                                                         const uint16_t *__restrict__ mask) {
    __shared__ float w[kPwMaxCin * CO];
    for (int i = threadIdx.x; i < cin * CO; i += kThreads) w[i] = bf16_to_f32(p[i]);
    __syncthreads();
    const unsigned long long t = static_cast<unsigned long long>(blockIdx.x) * kThreads + threadIdx.x;
    const unsigned v = static_cast<unsigned>(t >> cg_shift), c8 = static_cast<unsigned>(t) & ((1u << cg_shift) - 1);
    if (v >= l.nvox) return;
    const Vox o = decode(v, l);
    const long long pv = pidx(g, o.tile, o.ld, o.lh, o.lw);
    float gv[CO];
#pragma unroll
    for (int co = 0; co < CO; ++co) gv[co] = bf16_to_f32(dy[pv * CO + co]);
    uint32_t r[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int co = 0; co < CO; ++co) {
            s0 = fmaf(gv[co], w[(8 * c8 + 2 * e2) * CO + co], s0);
            s1 = fmaf(gv[co], w[(8 * c8 + 2 * e2 + 1) * CO + co], s1);
        }
        r[e2] = static_cast<uint32_t>(f32_to_bf16(s0)) | (static_cast<uint32_t>(f32_to_bf16(s1)) << 16);
    }
    if (mask) {      // backward of the ReLU that produced the layer input: keep dx where that input is positive
        const uint4 mv = *reinterpret_cast<const uint4 *>(mask + pv * cin + 8 * c8);
        r[0] &= positive_halves(mv.x); r[1] &= positive_halves(mv.y);
        r[2] &= positive_halves(mv.z); r[3] &= positive_halves(mv.w);
    }
    st_stream16(dx + pv * cin + 8 * c8, make_uint4(r[0], r[1], r[2], r[3]));
}

// dp[ci][co] = sum_v x[v][ci] * dy[v][co], db[co] = sum_v dy[v][co]: a block walks over a chunk of voxels
// with kThreads / (cin/8) voxel lanes x cin/8 channel groups (8 channels = one 16-byte load per thread);
// the voxel lanes are then added in lane order and the block's partial goes to ws[chunk][cin*CO (+CO)].
// DX: the same pass also writes the masked data gradient dx[v][ci] = [x[v][ci] > 0] * sum_co dy[v][co] * p[ci][co]
// (pointwise_small_dgrad_kernel's arithmetic with x itself as the mask): a thread already holds the 8 channels of
// x and the voxel's dy, so the layer input is read once for both gradients instead of twice.
template <int CO, bool DX>
__global__ __launch_bounds__(kThreads) void pointwise_small_wgrad_kernel(const uint16_t *__restrict__ x,
                                                                         const uint16_t *__restrict__ dy,
                                                                         float *__restrict__ part_w,
                                                                         float *__restrict__ part_b, Geo g, Lay l,
                                                                         int cin, int cg_shift, unsigned chunk_vox,
                                                                         const uint16_t *__restrict__ p,
                                                                         uint16_t *__restrict__ dx) {
    __shared__ float red[kThreads * (8 * CO)];
    __shared__ float w[DX ? kPwMaxCin * CO : 1];
    if (DX) {
        for (int i = threadIdx.x; i < cin * CO; i += kThreads) w[i] = bf16_to_f32(p[i]);
        __syncthreads();
    }
    const int cg = threadIdx.x & ((1 << cg_shift) - 1), vl = threadIdx.x >> cg_shift;
    const int nvl = kThreads >> cg_shift;
    float acc[8][CO], accb[CO];
#pragma unroll
    for (int co = 0; co < CO; ++co) {
        accb[co] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e][co] = 0.f;
    }
    const unsigned v0 = blockIdx.x * chunk_vox;
    unsigned v1 = v0 + chunk_vox;
    if (v1 > l.nvox) v1 = l.nvox;
    for (unsigned v = v0 + vl; v < v1; v += nvl) {
        const Vox o = decode(v, l);
        const long long pv = pidx(g, o.tile, o.ld, o.lh, o.lw);
        const uint4 q = *reinterpret_cast<const uint4 *>(x + pv * cin + 8 * cg);
        const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
        float gv[CO];
#pragma unroll
        for (int co = 0; co < CO; ++co) {
            gv[co] = bf16_to_f32(dy[pv * CO + co]);
            accb[co] += gv[co];
        }
        if (DX) {
            uint32_t r[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                float s0 = 0.f, s1 = 0.f;
#pragma unroll
                for (int co = 0; co < CO; ++co) {
                    s0 = fmaf(gv[co], w[(8 * cg + 2 * e2) * CO + co], s0);
                    s1 = fmaf(gv[co], w[(8 * cg + 2 * e2 + 1) * CO + co], s1);
                }
                r[e2] = static_cast<uint32_t>(f32_to_bf16(s0)) | (static_cast<uint32_t>(f32_to_bf16(s1)) << 16);
            }
            r[0] &= positive_halves(q.x); r[1] &= positive_halves(q.y);
            r[2] &= positive_halves(q.z); r[3] &= positive_halves(q.w);
            st_stream16(dx + pv * cin + 8 * cg, make_uint4(r[0], r[1], r[2], r[3]));
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float xv = __uint_as_float((e & 1) ? (qw[e >> 1] & 0xffff0000u) : (qw[e >> 1] << 16));
#pragma unroll
            for (int co = 0; co < CO; ++co) acc[e][co] = fmaf(xv, gv[co], acc[e][co]);
        }
    }
    // red[vl][ci][co]
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int co = 0; co < CO; ++co) red[(vl * cin + 8 * cg + e) * CO + co] = acc[e][co];
    __syncthreads();
    for (int i = threadIdx.x; i < cin * CO; i += kThreads) {
        float s = 0.f;
        for (int k = 0; k < nvl; ++k) s += red[k * cin * CO + i];
        part_w[static_cast<size_t>(blockIdx.x) * cin * CO + i] = s;
    }
    if (part_b) {
        __syncthreads();
        if (cg == 0) {
#pragma unroll
            for (int co = 0; co < CO; ++co) red[vl * CO + co] = accb[co];
        }
        __syncthreads();
        if (threadIdx.x < CO) {
            float s = 0.f;
            for (int k = 0; k < nvl; ++k) s += red[k * CO + threadIdx.x];
            part_b[static_cast<size_t>(blockIdx.x) * CO + threadIdx.x] = s;
        }
    }
}

void pointwise_wgrad_plan(unsigned nvox, int *nchunks, unsigned *chunk_vox) {
    unsigned cv = 4096;
    unsigned nc = (nvox + cv - 1) / cv;
    if (nc > 2048) { nc = 2048; cv = (nvox + nc - 1) / nc; nc = (nvox + cv - 1) / cv; }
    *nchunks = static_cast<int>(nc);
    *chunk_vox = cv;
}

void upconv_wgrad_plan(unsigned nvox, int cin, int cout, int *nchunks, unsigned *chunk_vox) {
    const size_t per_chunk = 8ull * cin * cout * sizeof(float);
    size_t cap = (256ull << 20) / per_chunk;
    if (cap < 1) cap = 1;
    if (cap > 4096) cap = 4096;
    size_t want = (nvox + 1023) / 1024;
    if (want < 1) want = 1;
    const unsigned nc = static_cast<unsigned>(want < cap ? want : cap);
    const unsigned cv = (nvox + nc - 1) / nc;
    *nchunks = static_cast<int>((nvox + cv - 1) / cv);
    *chunk_vox = cv;
}

void reduction_plan(unsigned nvox, int *nchunks, unsigned *chunk_vox) {
    unsigned cv = 8192;
    unsigned nc = (nvox + cv - 1) / cv;
    if (nc > 256) { nc = 256; cv = (nvox + nc - 1) / nc; nc = (nvox + cv - 1) / cv; }
    *nchunks = static_cast<int>(nc);
    *chunk_vox = cv;
}

}  // namespace

int make_coarse(const Geo &gf, Geo *gc) {
    if (((gf.flat ? 0 : gf.td) | gf.th | gf.tw) & 1) return SP_EGEOM;
    Geo o = gf;
    o.td = gf.flat ? gf.td : gf.td / 2; o.th = gf.th / 2; o.tw = gf.tw / 2;
    if ((!o.flat && o.td < o.halo) || o.th < o.halo || o.tw < o.halo) return SP_EGEOM;
    o.pd = o.td + 2 * o.halo; o.ph = o.th + 2 * o.halo; o.pw = o.tw + 2 * o.halo;
    o.tile_vox = 1LL * o.pd * o.ph * o.pw;
    o.int_vox = 1LL * o.td * o.th * o.tw;
    o.msg_vox = o.tile_vox - o.int_vox;
    *gc = o;
    return SP_OK;
}

#define SP3D_BY_DTYPE(call_bf16, call_f32) do { if (dt == SP_BF16) { call_bf16; } else { call_f32; } } while (0)

int launch_maxpool2(const void *Px, const void *Pdy, void *Pout, const Geo &gf, const Geo &gc, int c,
                    sp_dtype_t dt, bool backward, hipStream_t s, const void *Pskip) {
    if (1LL * gc.ntiles * gc.int_vox > 0xffffff00LL) return SP_EGEOM;
    if (dt == SP_BF16 && c % 8 == 0) {
        const Lay l = make_lay(gc, c / 8);
        const unsigned vpb = kThreads >> l.cshift;
        dim3 grid((l.nvox + vpb - 1) / vpb), block(kThreads);
#define SP3D_POOL8N(M, NW)                                                                                \
    hipLaunchKernelGGL((maxpool2_x8_kernel<M, NW>), grid, block, 0, s, static_cast<const uint16_t *>(Px), \
                       static_cast<const uint16_t *>(Pdy), static_cast<const uint16_t *>(Pskip),          \
                       static_cast<uint16_t *>(Pout), gf, gc, l, c)
#define SP3D_POOL8(M) do { if (gf.flat) SP3D_POOL8N(M, 4); else SP3D_POOL8N(M, 8); } while (0)
        if (backward && Pskip) SP3D_POOL8(kPoolBwdJoin);
        else if (backward) SP3D_POOL8(kPoolBwd);
        else SP3D_POOL8(kPoolFwd);
#undef SP3D_POOL8
#undef SP3D_POOL8N
        return record_hip(hipGetLastError());
    }
    const Lay l = make_lay(gc, c);
    const unsigned vpb = kThreads >> l.cshift;
    dim3 grid((l.nvox + vpb - 1) / vpb), block(kThreads);
#define SP3D_POOLN(E, B, NW)                                                                         \
    hipLaunchKernelGGL((maxpool2_kernel<E, B, NW>), grid, block, 0, s, static_cast<const E *>(Px),   \
                       static_cast<const E *>(Pdy), static_cast<const E *>(Pskip), static_cast<E *>(Pout), gf, gc, l, c)
#define SP3D_POOL(E, B) do { if (gf.flat) SP3D_POOLN(E, B, 4); else SP3D_POOLN(E, B, 8); } while (0)
    if (backward && Pskip) SP3D_BY_DTYPE(SP3D_POOL(uint16_t, kPoolBwdJoin), SP3D_POOL(float, kPoolBwdJoin));
    else if (backward) SP3D_BY_DTYPE(SP3D_POOL(uint16_t, kPoolBwd), SP3D_POOL(float, kPoolBwd));
    else SP3D_BY_DTYPE(SP3D_POOL(uint16_t, kPoolFwd), SP3D_POOL(float, kPoolFwd));
#undef SP3D_POOL
#undef SP3D_POOLN
    return record_hip(hipGetLastError());
}

int launch_upconv2_fwd(const void *Px, const void *u, const float *bias, void *Py, const Geo &gf,
                       const Geo &gc, int cin, int cout, sp_dtype_t dt, hipStream_t s) {
    if (upconv_mfma_supported(gf, gc, cin, cout, dt)) return launch_upconv_fwd_mfma(Px, u, bias, Py, gf, gc, cin, cout, s);
    if (1LL * gf.ntiles * gf.int_vox > 0xffffff00LL) return SP_EGEOM;
    const Lay l = make_lay(gf, cout);
    const unsigned vpb = kThreads >> l.cshift;
    dim3 grid((l.nvox + vpb - 1) / vpb), block(kThreads);
#define SP3D_UP(E)                                                                                   \
    hipLaunchKernelGGL(upconv2_fwd_kernel<E>, grid, block, 0, s, static_cast<const E *>(Px),         \
                       static_cast<const E *>(u), bias, static_cast<E *>(Py), gf, gc, l, cin, cout)
    SP3D_BY_DTYPE(SP3D_UP(uint16_t), SP3D_UP(float));
#undef SP3D_UP
    return record_hip(hipGetLastError());
}

int launch_upconv2_dgrad(const void *Pdy, const void *u, void *Pdx, const Geo &gf, const Geo &gc, int cin,
                         int cout, sp_dtype_t dt, hipStream_t s) {
    if (upconv_mfma_supported(gf, gc, cin, cout, dt)) return launch_upconv_dgrad_mfma(Pdy, u, Pdx, gf, gc, cin, cout, s);
    if (1LL * gf.ntiles * gf.int_vox > 0xffffff00LL) return SP_EGEOM;
    const Lay l = make_lay(gc, cin);
    const unsigned vpb = kThreads >> l.cshift;
    dim3 grid((l.nvox + vpb - 1) / vpb), block(kThreads);
#define SP3D_UPD(E)                                                                                  \
    hipLaunchKernelGGL(upconv2_dgrad_kernel<E>, grid, block, 0, s, static_cast<const E *>(Pdy),      \
                       static_cast<const E *>(u), static_cast<E *>(Pdx), gf, gc, l, cin, cout)
    if (dt == SP_BF16 && cout % 8 == 0) {
        hipLaunchKernelGGL(upconv2_dgrad_bf16x8_kernel, grid, block, 0, s, static_cast<const uint16_t *>(Pdy),
                           static_cast<const uint16_t *>(u), static_cast<uint16_t *>(Pdx), gf, gc, l, cin, cout);
        return record_hip(hipGetLastError());
    }
    SP3D_BY_DTYPE(SP3D_UPD(uint16_t), SP3D_UPD(float));
#undef SP3D_UPD
    return record_hip(hipGetLastError());
}

size_t upconv2_wgrad_ws_bytes(const Geo &gf, const Geo &gc, int cin, int cout, sp_dtype_t dt) {
    if (upconv_mfma_supported(gf, gc, cin, cout, dt)) return upconv_wgrad_mfma_ws_bytes(gc, cin, cout);
    int ncw; unsigned cvw;
    upconv_wgrad_plan(static_cast<unsigned>(1LL * gc.ntiles * gc.int_vox), cin, cout, &ncw, &cvw);
    int ncb; unsigned cvb;
    reduction_plan(static_cast<unsigned>(1LL * gf.ntiles * gf.int_vox), &ncb, &cvb);
    return (static_cast<size_t>(ncw) * (gf.flat ? 4 : 8) * cin * cout + static_cast<size_t>(ncb) * cout) * sizeof(float);
}

int launch_upconv2_wgrad(const void *Px, const void *Pdy, float *du, float *db, const Geo &gf, const Geo &gc,
                         int cin, int cout, sp_dtype_t dt, void *ws, hipStream_t s) {
    if (upconv_mfma_supported(gf, gc, cin, cout, dt))
        return launch_upconv_wgrad_mfma(Px, Pdy, du, db, gf, gc, cin, cout, ws, s);
    if (1LL * gf.ntiles * gf.int_vox > 0xffffff00LL) return SP_EGEOM;
    const Lay lc = make_lay(gc, cout), lf = make_lay(gf, cout);
    int ncw, ncb; unsigned cvw, cvb;
    upconv_wgrad_plan(lc.nvox, cin, cout, &ncw, &cvw);
    reduction_plan(lf.nvox, &ncb, &cvb);
    float *part_w = static_cast<float *>(ws);
    const int nk = gf.flat ? 4 : 8;          // window positions = taps of u
    float *part_b = part_w + static_cast<size_t>(ncw) * nk * cin * cout;
    const int cw = cout < kThreads ? cout : kThreads;
    const int zg = (cout + cw - 1) / cw;
    dim3 block(kThreads), gw_(nk * cin, ncw, zg), gb_(1, ncb, zg);
    int co8_shift = -1;
    if (dt == SP_BF16 && cout % 8 == 0 && cout <= 8 * kThreads && ((cout / 8) & (cout / 8 - 1)) == 0) {
        co8_shift = 0;
        while ((1 << co8_shift) < cout / 8) ++co8_shift;
    }
    if (co8_shift >= 0) {
        const int cipb = kThreads >> co8_shift;
        hipLaunchKernelGGL(upconv2_wgrad_bf16x8_kernel, dim3((cin + cipb - 1) / cipb, ncw), block, 0, s,
                           static_cast<const uint16_t *>(Px), static_cast<const uint16_t *>(Pdy), part_w, gf, gc, lc,
                           cin, cout, co8_shift, cvw);
        if (db)
            hipLaunchKernelGGL(bsum_kernel<uint16_t>, gb_, block, 0, s, static_cast<const uint16_t *>(Pdy), part_b,
                               gf, lf, cout, cw, cvb);
        int rc2 = record_hip(hipGetLastError());
        if (rc2 != SP_OK) return rc2;
        rc2 = launch_reduce_partials(part_w, du, ncw, 1LL * nk * cin * cout, s);
        if (rc2 != SP_OK) return rc2;
        if (db) rc2 = launch_reduce_partials(part_b, db, ncb, cout, s);
        return rc2;
    }
#define SP3D_UPW(E)                                                                                  \
    do {                                                                                             \
        hipLaunchKernelGGL(upconv2_wgrad_kernel<E>, gw_, block, 0, s, static_cast<const E *>(Px),    \
                           static_cast<const E *>(Pdy), part_w, gf, gc, lc, cin, cout, cw, cvw);     \
        if (db)                                                                                      \
            hipLaunchKernelGGL(bsum_kernel<E>, gb_, block, 0, s, static_cast<const E *>(Pdy), part_b, gf, lf, \
                               cout, cw, cvb);                                                       \
    } while (0)
    SP3D_BY_DTYPE(SP3D_UPW(uint16_t), SP3D_UPW(float));
#undef SP3D_UPW
    int rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    rc = launch_reduce_partials(part_w, du, ncw, 1LL * nk * cin * cout, s);
    if (rc != SP_OK) return rc;
    if (db) rc = launch_reduce_partials(part_b, db, ncb, cout, s);
    return rc;
}

int launch_add(const void *Pa, const void *Pb, void *Pout, size_t elems, sp_dtype_t dt, hipStream_t s) {
    if (dt == SP_BF16 && elems % 8 == 0 && (elems / 8 + kThreads - 1) / kThreads <= 0x7fffffffULL) {
        const size_t nvec = elems / 8;
        hipLaunchKernelGGL(add_bf16x8_kernel, dim3(static_cast<unsigned>((nvec + kThreads - 1) / kThreads)),
                           dim3(kThreads), 0, s, static_cast<const uint4 *>(Pa), static_cast<const uint4 *>(Pb),
                           static_cast<uint4 *>(Pout), nvec);
        return record_hip(hipGetLastError());
    }
    const size_t blocks = (elems + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffULL) return SP_EGEOM;
    dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    SP3D_BY_DTYPE(hipLaunchKernelGGL(add_kernel<uint16_t>, grid, block, 0, s, static_cast<const uint16_t *>(Pa),
                                     static_cast<const uint16_t *>(Pb), static_cast<uint16_t *>(Pout), elems),
                  hipLaunchKernelGGL(add_kernel<float>, grid, block, 0, s, static_cast<const float *>(Pa),
                                     static_cast<const float *>(Pb), static_cast<float *>(Pout), elems));
    return record_hip(hipGetLastError());
}

int launch_concat(const void *Pa, int ca, const void *Pb, int cb, void *Pc, size_t voxels, sp_dtype_t dt,
                  bool split, hipStream_t s) {
    if (dt == SP_BF16 && ca % 8 == 0 && cb % 8 == 0) {
        const size_t total8 = voxels * ((ca + cb) / 8);
        const size_t blocks8 = (total8 + kThreads - 1) / kThreads;
        if (blocks8 > 0x7fffffffULL) return SP_EGEOM;
        dim3 grid8(static_cast<unsigned>(blocks8)), block8(kThreads);
        uint4 *pa = static_cast<uint4 *>(const_cast<void *>(Pa)), *pb = static_cast<uint4 *>(const_cast<void *>(Pb));
        if (split)
            hipLaunchKernelGGL(concat_x8_kernel<true>, grid8, block8, 0, s, pa, ca / 8, pb, cb / 8,
                               static_cast<uint4 *>(Pc), total8);
        else
            hipLaunchKernelGGL(concat_x8_kernel<false>, grid8, block8, 0, s, pa, ca / 8, pb, cb / 8,
                               static_cast<uint4 *>(Pc), total8);
        return record_hip(hipGetLastError());
    }
    const size_t total = voxels * (ca + cb);
    const size_t blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffULL) return SP_EGEOM;
    dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
#define SP3D_CAT(E, S)                                                                               \
    hipLaunchKernelGGL((concat_kernel<E, S>), grid, block, 0, s, static_cast<E *>(const_cast<void *>(Pa)), ca, \
                       static_cast<E *>(const_cast<void *>(Pb)), cb, static_cast<E *>(Pc), total)
    if (split) SP3D_BY_DTYPE(SP3D_CAT(uint16_t, true), SP3D_CAT(float, true));
    else SP3D_BY_DTYPE(SP3D_CAT(uint16_t, false), SP3D_CAT(float, false));
#undef SP3D_CAT
    return record_hip(hipGetLastError());
}

bool pointwise_small_supported(const Geo &g, int cin, int cout, sp_dtype_t dt) {
    if (dt != SP_BF16 || cout < 1 || cout > 4 || cin % 8 != 0 || cin > kPwMaxCin) return false;
    const int cg = cin / 8;
    return (cg & (cg - 1)) == 0 && 1LL * g.ntiles * g.int_vox <= 0xffffff00LL;
}

#define SP3D_BY_CO(KERNEL, ...)                                                                      \
    switch (cout) {                                                                                  \
    case 1: hipLaunchKernelGGL(KERNEL<1>, __VA_ARGS__); break;                                       \
    case 2: hipLaunchKernelGGL(KERNEL<2>, __VA_ARGS__); break;                                       \
    case 3: hipLaunchKernelGGL(KERNEL<3>, __VA_ARGS__); break;                                       \
    default: hipLaunchKernelGGL(KERNEL<4>, __VA_ARGS__); break;                                      \
    }

int launch_pointwise_small_fwd(const void *Px, const void *p, const float *bias, void *Py, const Geo &g, int cin,
                               int cout, bool relu, hipStream_t s) {
    const Lay l = make_lay(g, 1);
    dim3 grid((l.nvox + kThreads - 1) / kThreads), block(kThreads);
    SP3D_BY_CO(pointwise_small_fwd_kernel, grid, block, 0, s, static_cast<const uint16_t *>(Px),
               static_cast<const uint16_t *>(p), bias, static_cast<uint16_t *>(Py), g, l, cin, relu ? 1 : 0)
    return record_hip(hipGetLastError());
}

int launch_pointwise_small_dgrad(const void *Pdy, const void *p, void *Pdx, const Geo &g, int cin, int cout,
                                 hipStream_t s, const void *Pmask) {
    const Lay l = make_lay(g, 1);
    int cg_shift = 0;
    while ((1 << cg_shift) < cin / 8) ++cg_shift;
    const unsigned long long threads = static_cast<unsigned long long>(l.nvox) << cg_shift;
    const unsigned long long blocks = (threads + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffULL) return SP_EGEOM;
    dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    SP3D_BY_CO(pointwise_small_dgrad_kernel, grid, block, 0, s, static_cast<const uint16_t *>(Pdy),
               static_cast<const uint16_t *>(p), static_cast<uint16_t *>(Pdx), g, l, cin, cg_shift,
               static_cast<const uint16_t *>(Pmask))
    return record_hip(hipGetLastError());
}

size_t pointwise_small_wgrad_ws_bytes(const Geo &g, int cin, int cout) {
    int nc; unsigned cv;
    pointwise_wgrad_plan(static_cast<unsigned>(1LL * g.ntiles * g.int_vox), &nc, &cv);
    return static_cast<size_t>(nc) * (cin * cout + cout) * sizeof(float);
}

int launch_pointwise_small_wgrad(const void *Px, const void *Pdy, float *dp, float *db, const Geo &g, int cin,
                                 int cout, void *ws, hipStream_t s, const void *p, void *Pdx) {
    const Lay l = make_lay(g, 1);
    int nc; unsigned cv;
    pointwise_wgrad_plan(l.nvox, &nc, &cv);
    float *part_w = static_cast<float *>(ws);
    float *part_b = db ? part_w + static_cast<size_t>(nc) * cin * cout : nullptr;
    int cg_shift = 0;
    while ((1 << cg_shift) < cin / 8) ++cg_shift;
    dim3 grid(nc), block(kThreads);
#define SP3D_WG(CO)                                                                                            \
    case CO:                                                                                                   \
        if (Pdx)                                                                                               \
            hipLaunchKernelGGL((pointwise_small_wgrad_kernel<CO, true>), grid, block, 0, s,                    \
                               static_cast<const uint16_t *>(Px), static_cast<const uint16_t *>(Pdy), part_w,  \
                               part_b, g, l, cin, cg_shift, cv, static_cast<const uint16_t *>(p),              \
                               static_cast<uint16_t *>(Pdx));                                                  \
        else                                                                                                   \
            hipLaunchKernelGGL((pointwise_small_wgrad_kernel<CO, false>), grid, block, 0, s,                   \
                               static_cast<const uint16_t *>(Px), static_cast<const uint16_t *>(Pdy), part_w,  \
                               part_b, g, l, cin, cg_shift, cv, nullptr, nullptr);                             \
        break;
    switch (cout) {
        SP3D_WG(1) SP3D_WG(2) SP3D_WG(3) SP3D_WG(4)
    default: return SP_EUNSUPPORTED;
    }
#undef SP3D_WG
    int rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    rc = launch_reduce_partials(part_w, dp, nc, 1LL * cin * cout, s);
    if (rc != SP_OK) return rc;
    if (db) rc = launch_reduce_partials(part_b, db, nc, cout, s);
    return rc;
}
#undef SP3D_BY_CO

}  // namespace sp3d
