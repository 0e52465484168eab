// Direct (non-MFMA) convolution kernels on padded tiles.  They serve every channel count and both
// dtypes: the fp32 configuration, odd channel counts, and anything the MFMA kernels do not cover.
// fp32 accumulation with fused multiply-add, taps in (kd,kh,kw) order, input channels innermost.
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

// One thread per (voxel of the output box, output channel).  With DGRAD the taps are mirrored and the weight
// tensor is read as w[tap][ko][ki] (ko = this kernel's output channel = the layer's input channel).
// KS = kernel extent per axis: 3 (the 3x3x3 convolution) or 1 (the 1x1x1 classifier); in the 2-D variant
// (g.flat) the extent along D is 1 and the box does not grow along D.
// The threads cover the interior grown by g.grow on every side; a thread whose voxel lies beyond a side on
// which its tile has no neighbour (beyond the volume) has nothing to do.
template <typename E, bool DGRAD, int KS>
__global__ __launch_bounds__(kThreads) void conv_direct_kernel(const E *__restrict__ Pin,
                                                               const E *__restrict__ w,
                                                               const float *__restrict__ bias,
                                                               E *__restrict__ Pout, Geo g, int ki,
                                                               int ko, int relu, long long total,
                                                               const E *__restrict__ mask) {
    const long long idx = 1LL * blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int co = static_cast<int>(idx % ko);
    const long long v = idx / ko;                       // voxel of the grown boxes of all tiles
    const int gd_ = grow_d(g);
    const int ed = g.td + 2 * gd_, eh = g.th + 2 * g.grow, ew = g.tw + 2 * g.grow;
    const long long box_vox = 1LL * ed * eh * ew;
    const long long tile = v / box_vox;
    const unsigned r = static_cast<unsigned>(v % box_vox);
    const unsigned ehw = static_cast<unsigned>(eh) * ew;
    // padded coordinates of the output voxel
    const int pd = static_cast<int>(r / ehw) + g.halo - gd_, ph = static_cast<int>((r % ehw) / ew) + g.halo - g.grow,
              pw = static_cast<int>(r % ew) + g.halo - g.grow;
    if (g.grow > 0) {
        const int tc = static_cast<int>(tile % g.gw), tb = static_cast<int>((tile / g.gw) % g.gh),
                  ta = static_cast<int>((tile / (1LL * g.gw * g.gh)) % g.gd);
        if ((pd < g.halo && ta == 0) || (pd >= g.halo + g.td && ta == g.gd - 1) || (ph < g.halo && tb == 0) ||
            (ph >= g.halo + g.th && tb == g.gh - 1) || (pw < g.halo && tc == 0) ||
            (pw >= g.halo + g.tw && tc == g.gw - 1))
            return;
    }
    const long long base = tile * g.tile_vox;
    float acc = bias ? bias[co] : 0.f;
    constexpr int O = KS / 2;         // tap k reads the input voxel at output coordinate + k - O
    const int KD = g.flat ? 1 : KS, OD = KD / 2;
    for (int kd = 0; kd < KD; ++kd)
        for (int kh = 0; kh < KS; ++kh)
            for (int kw = 0; kw < KS; ++kw) {
                const long long pv = base + (1LL * (pd + kd - OD) * g.ph + ph + kh - O) * g.pw + pw + kw - O;
                const E *xin = Pin + pv * ki;
                const int tap = DGRAD ? ((KD - 1 - kd) * KS + (KS - 1 - kh)) * KS + (KS - 1 - kw)
                                      : (kd * KS + kh) * KS + kw;
                if (DGRAD) {
                    const E *wt = w + (1LL * tap * ko + co) * ki;      // w[tap][ci=co][co'=c]
                    for (int c = 0; c < ki; ++c) acc = fmaf(ldf<E>(xin, c), ldf<E>(wt, c), acc);
                } else {
                    const E *wt = w + 1LL * tap * ki * ko + co;        // w[tap][c][co]
                    for (int c = 0; c < ki; ++c)
                        acc = fmaf(ldf<E>(xin, c), ldf<E>(wt, 1LL * c * ko), acc);
                }
            }
    if (relu && acc < 0.f) acc = 0.f;
    const long long ov = base + (1LL * pd * g.ph + ph) * g.pw + pw;
    if (mask && !(ldf<E>(mask, ov * ko + co) > 0.f)) acc = 0.f;      // backward of the ReLU that produced the input
    stf<E>(Pout, ov * ko + co, acc);
}

// Weight gradient, stage 1.  Block (tap*cin + ci, chunk, co-group): threads are laid out as
// [voxel lane][co]; each thread sums its voxels of the chunk in index order, then the voxel lanes
// are added in lane order by one thread per co.  Partial sums go to ws[chunk][tap][ci][co].
template <typename E, int KS>
__global__ __launch_bounds__(kThreads) void wgrad_direct_kernel(const E *__restrict__ Px,
                                                                const E *__restrict__ Pdz,
                                                                float *__restrict__ part, Geo g,
                                                                int cin, int cout, int cw,
                                                                long long chunk_vox,
                                                                long long total_vox) {
    __shared__ float red[kThreads];
    const int tapci = blockIdx.x, chunk = blockIdx.y;
    const int tap = tapci / cin, ci = tapci % cin;
    const int O = g.halo - KS / 2;    // tap k reads padded coordinate (interior coordinate + k + O)
    // 2-D variant: KS * KS taps, all in the voxel's own slice
    const int kd = g.flat ? g.halo : tap / (KS * KS) + O, kh = (tap / KS) % KS + O, kw = tap % KS + O;
    const int nvl = kThreads / cw;
    const int col = threadIdx.x % cw, vl = threadIdx.x / cw;
    const int co = blockIdx.z * cw + col;
    const unsigned thw = static_cast<unsigned>(g.th) * g.tw;
    float acc = 0.f;
    long long v1 = (chunk + 1LL) * chunk_vox;
    if (v1 > total_vox) v1 = total_vox;
    if (vl < nvl && co < cout) {
        for (long long v = 1LL * chunk * chunk_vox + vl; v < v1; v += nvl) {
            const long long tile = v / g.int_vox;
            const unsigned r = static_cast<unsigned>(v % g.int_vox);
            const unsigned ld = r / thw, lh = (r % thw) / g.tw, lw = r % g.tw;
            const long long base = tile * g.tile_vox;
            const long long xv = base + (1LL * (ld + kd) * g.ph + lh + kh) * g.pw + lw + kw;
            const long long zv = base + (1LL * (ld + g.halo) * g.ph + lh + g.halo) * g.pw + lw + g.halo;
            acc = fmaf(ldf<E>(Px, xv * cin + ci), ldf<E>(Pdz, zv * cout + co), acc);
        }
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (vl == 0 && co < cout) {
        float s = 0.f;
        for (int l = 0; l < nvl; ++l) s += red[l * cw + col];
        part[(1LL * chunk * gridDim.x + tapci) * cout + co] = s;
    }
}

// Bias gradient, stage 1: block = chunk of interior voxels, thread layout as above.
template <typename E>
__global__ __launch_bounds__(kThreads) void bgrad_direct_kernel(const E *__restrict__ Pdz,
                                                                float *__restrict__ part, Geo g,
                                                                int cout, int cw, long long chunk_vox,
                                                                long long total_vox) {
    __shared__ float red[kThreads];
    const int chunk = blockIdx.y;
    const int nvl = kThreads / cw;
    const int col = threadIdx.x % cw, vl = threadIdx.x / cw;
    const int co = blockIdx.z * cw + col;
    const unsigned thw = static_cast<unsigned>(g.th) * g.tw;
    float acc = 0.f;
    long long v1 = (chunk + 1LL) * chunk_vox;
    if (v1 > total_vox) v1 = total_vox;
    if (vl < nvl && co < cout) {
        for (long long v = 1LL * chunk * chunk_vox + vl; v < v1; v += nvl) {
            const long long tile = v / g.int_vox;
            const unsigned r = static_cast<unsigned>(v % g.int_vox);
            const unsigned ld = r / thw, lh = (r % thw) / g.tw, lw = r % g.tw;
            const long long zv = tile * g.tile_vox +
                                 (1LL * (ld + g.halo) * g.ph + lh + g.halo) * g.pw + lw + g.halo;
            acc += ldf<E>(Pdz, zv * cout + co);
        }
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (vl == 0 && co < cout) {
        float s = 0.f;
        for (int l = 0; l < nvl; ++l) s += red[l * cw + col];
        part[1LL * chunk * cout + co] = s;
    }
}

}  // namespace

// Stage 2 (shared with the MFMA weight-gradient kernel): out[e] = sum_s part[s][e] in order of s.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ part,
                                                              float *__restrict__ out, int nparts,
                                                              long long n) {
    const long long e = 1LL * blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    float s = 0.f;
    for (int p = 0; p < nparts; ++p) s += part[1LL * p * n + e];
    out[e] = s;
}

// Same sum for few outputs and many partials (one serial chain per output would be latency-bound): a block
// per output; thread t adds the partials t, t + 256, ... in order, then the 256 thread sums are combined
// by a fixed binary tree.  The grouping depends only on nparts, so the result is still reproducible.
__global__ __launch_bounds__(256) void reduce_partials_wide_kernel(const float *__restrict__ part,
                                                                   float *__restrict__ out, int nparts,
                                                                   long long n) {
    __shared__ float red[256];
    const long long e = blockIdx.x;
    float s = 0.f;
    for (int p = threadIdx.x; p < nparts; p += 256) s += part[1LL * p * n + e];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[e] = red[0];
}

int launch_reduce_partials(const float *part, float *out, int nparts, long long n, hipStream_t s) {
    if (nparts >= 512 && n <= 16384) {
        hipLaunchKernelGGL(reduce_partials_wide_kernel, dim3(static_cast<unsigned>(n)), dim3(256), 0, s, part, out,
                           nparts, n);
        return record_hip(hipGetLastError());
    }
    dim3 grid(static_cast<unsigned>((n + 255) / 256)), block(256);
    hipLaunchKernelGGL(reduce_partials_kernel, grid, block, 0, s, part, out, nparts, n);
    return record_hip(hipGetLastError());
}

int launch_conv_direct(const void *Pin, const void *w, const float *bias, void *Pout, const Geo &g,
                       int ki, int ko, sp_dtype_t dt, bool relu, bool dgrad, hipStream_t s, int ks,
                       const void *mask) {
    const long long total = 1LL * g.ntiles * (g.td + 2 * grow_d(g)) * (g.th + 2 * g.grow) * (g.tw + 2 * g.grow) * ko;
    const long long blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return SP_EGEOM;
    dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
#define SP3D_LAUNCH(E, DG, KS)                                                                         \
    hipLaunchKernelGGL((conv_direct_kernel<E, DG, KS>), grid, block, 0, s, static_cast<const E *>(Pin), \
                       static_cast<const E *>(w), bias, static_cast<E *>(Pout), g, ki, ko,             \
                       relu ? 1 : 0, total, static_cast<const E *>(mask))
#define SP3D_LAUNCH_KS(E, DG) do { if (ks == 1) SP3D_LAUNCH(E, DG, 1); else SP3D_LAUNCH(E, DG, 3); } while (0)
    if (dt == SP_BF16) {
        if (dgrad) SP3D_LAUNCH_KS(uint16_t, true); else SP3D_LAUNCH_KS(uint16_t, false);
    } else {
        if (dgrad) SP3D_LAUNCH_KS(float, true); else SP3D_LAUNCH_KS(float, false);
    }
#undef SP3D_LAUNCH_KS
#undef SP3D_LAUNCH
    return record_hip(hipGetLastError());
}

// chunking of the voxel reduction for the direct weight gradient
static void wgrad_direct_plan(const Geo &g, int *nchunks, long long *chunk_vox) {
    const long long total = 1LL * g.ntiles * g.int_vox;
    long long cv = 8192;
    long long nc = (total + cv - 1) / cv;
    if (nc > 256) { nc = 256; cv = (total + nc - 1) / nc; nc = (total + cv - 1) / cv; }
    *nchunks = static_cast<int>(nc);
    *chunk_vox = cv;
}

size_t wgrad_direct_ws_bytes(const Geo &g, int cin, int cout, int ks) {
    int nc; long long cv;
    wgrad_direct_plan(g, &nc, &cv);
    const size_t taps = static_cast<size_t>(g.flat ? 1 : ks) * ks * ks;
    return (static_cast<size_t>(nc) * taps * cin * cout + static_cast<size_t>(nc) * cout) * sizeof(float);
}

int launch_wgrad_direct(const void *Px, const void *Pdz, float *dw, float *db, const Geo &g, int cin,
                        int cout, sp_dtype_t dt, void *ws, hipStream_t s, int ks) {
    int nc; long long cv;
    wgrad_direct_plan(g, &nc, &cv);
    const long long total = 1LL * g.ntiles * g.int_vox;
    const int taps = (g.flat ? 1 : ks) * ks * ks;
    float *part_w = static_cast<float *>(ws);
    float *part_b = part_w + static_cast<size_t>(nc) * taps * cin * cout;
    const int cw = cout < kThreads ? cout : kThreads;
    const int zg = (cout + cw - 1) / cw;
    if (nc > 65535 || zg > 65535) return SP_EUNSUPPORTED;
    dim3 block(kThreads), gw_(taps * cin, nc, zg), gb_(1, nc, zg);
    if (dt == SP_BF16) {
        if (ks == 1)
            hipLaunchKernelGGL((wgrad_direct_kernel<uint16_t, 1>), gw_, block, 0, s,
                               static_cast<const uint16_t *>(Px), static_cast<const uint16_t *>(Pdz),
                               part_w, g, cin, cout, cw, cv, total);
        else
            hipLaunchKernelGGL((wgrad_direct_kernel<uint16_t, 3>), gw_, block, 0, s,
                               static_cast<const uint16_t *>(Px), static_cast<const uint16_t *>(Pdz),
                               part_w, g, cin, cout, cw, cv, total);
        if (db)
            hipLaunchKernelGGL(bgrad_direct_kernel<uint16_t>, gb_, block, 0, s,
                               static_cast<const uint16_t *>(Pdz), part_b, g, cout, cw, cv, total);
    } else {
        if (ks == 1)
            hipLaunchKernelGGL((wgrad_direct_kernel<float, 1>), gw_, block, 0, s,
                               static_cast<const float *>(Px), static_cast<const float *>(Pdz), part_w, g,
                               cin, cout, cw, cv, total);
        else
            hipLaunchKernelGGL((wgrad_direct_kernel<float, 3>), gw_, block, 0, s,
                               static_cast<const float *>(Px), static_cast<const float *>(Pdz), part_w, g,
                               cin, cout, cw, cv, total);
        if (db)
            hipLaunchKernelGGL(bgrad_direct_kernel<float>, gb_, block, 0, s,
                               static_cast<const float *>(Pdz), part_b, g, cout, cw, cv, total);
    }
    int rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    rc = launch_reduce_partials(part_w, dw, nc, 1LL * taps * cin * cout, s);
    if (rc != SP_OK) return rc;
    if (db) rc = launch_reduce_partials(part_b, db, nc, cout, s);
    return rc;
}

}  // namespace sp3d
