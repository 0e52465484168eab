// Segmentation loss on padded tiles: soft Dice + cross-entropy over the class logits, and its gradient
// with respect to the logits.  Two passes over the voxels, both bound by HBM traffic (a few bytes per voxel):
//
//   pass 1  per class c:  I_c = sum_v p[v,c] y[v,c],  P_c = sum_v p[v,c],  Y_c = sum_v y[v,c];  N = -sum_v log p[v, label v]
//           p = softmax of the voxel's logits, y = one-hot label.  The sums run over the interiors of ALL tiles
//           (the cross-tile reduction of the path): per-thread fp32 sums, a fixed tree per block, then the
//           fixed-order second stage shared with the weight gradients, so the result is reproducible.
//   pass 2  loss = w_dice (1 - mean_c (2 I_c + eps) / (P_c + Y_c + eps)) + w_ce N / V
//           dz[v,k] = p_k (g_k - sum_c g_c p_c) + w_ce (p_k - y_k) / V,
//           g_c = -(w_dice / C) (2 y_c S_c - (2 I_c + eps)) / S_c^2,  S_c = P_c + Y_c + eps
//
// Labels are a one-channel padded tensor of the logits' dtype holding the class index of every voxel.
#include "common.h"

namespace sp3d {

namespace {

constexpr int kThreads = 256;
constexpr unsigned kChunk = 8192;         // voxels per block in pass 1

template <typename E> __device__ __forceinline__ float widen(E v);
template <> __device__ __forceinline__ float widen<float>(float v) { return v; }
template <> __device__ __forceinline__ float widen<uint16_t>(uint16_t v) { return bf16_to_f32(v); }
template <typename E> __device__ __forceinline__ E narrow(float v);
template <> __device__ __forceinline__ float narrow<float>(float v) { return v; }
template <> __device__ __forceinline__ uint16_t narrow<uint16_t>(float v) { return f32_to_bf16(v); }

// A thread works on VPT consecutive voxels of a W row (VPT divides the tile's W extent, so a group never
// leaves its row) and moves their records as one block: with 3 classes of bf16 a voxel is 6 bytes, and
// 8 voxels make three 16-byte accesses per lane where single voxels would make 2-byte ones.  The copies
// below have only the element's alignment; the compiler turns them into full-width global accesses.
template <typename E, int N> struct __attribute__((packed, aligned(sizeof(E)))) Rec { E e[N]; };
template <typename E, int N> __device__ __forceinline__ void load_rec(const E *p, Rec<E, N> &r) {
    __builtin_memcpy(&r, p, sizeof(r));
}
template <typename E, int N> __device__ __forceinline__ void store_rec(E *p, const Rec<E, N> &r) {
    __builtin_memcpy(p, &r, sizeof(r));
}

struct LossGeo {
    Geo g;
    unsigned nvox;                 // interior voxels of all tiles
    FastDiv int_vox, hw, w;
};

__device__ __forceinline__ long long padded_index(const LossGeo &l, unsigned v) {
    const unsigned tile = fdiv(v, l.int_vox), r = fmod_(v, tile, l.int_vox);
    const unsigned ld = fdiv(r, l.hw), q = fmod_(r, ld, l.hw);
    const unsigned lh = fdiv(q, l.w), lw = fmod_(q, lh, l.w);
    return tile * l.g.tile_vox + (1LL * (ld + 1) * l.g.ph + lh + 1) * l.g.pw + lw + 1;
}

// softmax of one voxel from its stored logits; returns the label (clamped into range: the host cannot check
// every voxel)
template <typename E, int C>
__device__ __forceinline__ int voxel_softmax(const E *zr, E labv, float (&p)[C]) {
    float m = -3.0e38f;
#pragma unroll
    for (int c = 0; c < C; ++c) { p[c] = widen<E>(zr[c]); m = fmaxf(m, p[c]); }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < C; ++c) { p[c] = __expf(p[c] - m); s += p[c]; }
    const float inv = 1.f / s;
#pragma unroll
    for (int c = 0; c < C; ++c) p[c] *= inv;
    const int k = static_cast<int>(widen<E>(labv));
    return k < 0 ? 0 : (k >= C ? C - 1 : k);
}

// pass 1: part[block][0..C) = I, [C..2C) = P, [2C..3C) = Y, [3C] = N
template <typename E, int C, int VPT>
__global__ __launch_bounds__(kThreads) void loss_stats_kernel(const E *__restrict__ z, const E *__restrict__ lab,
                                                              float *__restrict__ part, LossGeo l) {
    __shared__ float red[kThreads];
    float acc[3 * C + 1];
#pragma unroll
    for (int i = 0; i < 3 * C + 1; ++i) acc[i] = 0.f;
    const unsigned v0 = blockIdx.x * kChunk;
    const unsigned v1 = v0 + kChunk < l.nvox ? v0 + kChunk : l.nvox;
    for (unsigned v = v0 + threadIdx.x * VPT; v < v1; v += kThreads * VPT) {   // kChunk and nvox are multiples of VPT
        const long long pv = padded_index(l, v);
        Rec<E, VPT * C> zr;
        Rec<E, VPT> lr;
        load_rec(z + pv * C, zr);
        load_rec(lab + pv, lr);
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            float p[C];
            const int k = voxel_softmax<E, C>(zr.e + i * C, lr.e[i], p);
#pragma unroll
            for (int c = 0; c < C; ++c) {
                acc[C + c] += p[c];
                if (c == k) { acc[c] += p[c]; acc[2 * C + c] += 1.f; acc[3 * C] -= __logf(fmaxf(p[c], 1e-38f)); }
            }
        }
    }
    // a fixed tree per statistic: butterfly inside each wave, then the four wave sums in wave order
#pragma unroll
    for (int i = 0; i < 3 * C + 1; ++i) {
        float v = acc[i];
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m);
        acc[i] = v;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < 3 * C + 1; ++i) red[wave * (3 * C + 1) + i] = acc[i];
    }
    __syncthreads();
    if (threadIdx.x < 3 * C + 1) {
        float t = 0.f;
        for (int w = 0; w < kThreads / 64; ++w) t += red[w * (3 * C + 1) + threadIdx.x];
        part[static_cast<size_t>(blockIdx.x) * (3 * C + 1) + threadIdx.x] = t;
    }
}

// pass 2: gradient (dz may be null) and the loss value (written by block 0)
template <typename E, int C, int VPT>
__global__ __launch_bounds__(kThreads) void loss_grad_kernel(const E *__restrict__ z, const E *__restrict__ lab,
                                                             const float *__restrict__ stats, E *__restrict__ dz,
                                                             float *__restrict__ loss, LossGeo l, float w_dice,
                                                             float w_ce, float eps) {
    float S[C], T[C];          // S_c = P_c + Y_c + eps, T_c = 2 I_c + eps
    float dice = 0.f;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        S[c] = stats[C + c] + stats[2 * C + c] + eps;
        T[c] = 2.f * stats[c] + eps;
        dice += T[c] / S[c];
    }
    const float invV = 1.f / static_cast<float>(l.nvox);
    if (loss && blockIdx.x == 0 && threadIdx.x == 0)
        loss[0] = w_dice * (1.f - dice / C) + w_ce * stats[3 * C] * invV;
    if (!dz) return;
    const unsigned long long v64 = (static_cast<unsigned long long>(blockIdx.x) * kThreads + threadIdx.x) * VPT;
    if (v64 >= l.nvox) return;
    const long long pv = padded_index(l, static_cast<unsigned>(v64));
    Rec<E, VPT * C> zr, out;
    Rec<E, VPT> lr;
    load_rec(z + pv * C, zr);
    load_rec(lab + pv, lr);
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        float p[C];
        const int k = voxel_softmax<E, C>(zr.e + i * C, lr.e[i], p);
        float g[C], gp = 0.f;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const float y = c == k ? 1.f : 0.f;
            g[c] = -(w_dice / C) * (2.f * y * S[c] - T[c]) / (S[c] * S[c]);
            gp += g[c] * p[c];
        }
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const float y = c == k ? 1.f : 0.f;
            out.e[i * C + c] = narrow<E>(p[c] * (g[c] - gp) + w_ce * (p[c] - y) * invV);
        }
    }
    store_rec(dz + pv * C, out);
}

LossGeo make_loss_geo(const Geo &g) {
    LossGeo l;
    l.g = g;
    l.nvox = static_cast<unsigned>(1LL * g.ntiles * g.int_vox);
    l.int_vox = make_fastdiv(static_cast<uint32_t>(g.int_vox));
    l.hw = make_fastdiv(static_cast<uint32_t>(g.th) * g.tw);
    l.w = make_fastdiv(g.tw);
    return l;
}

template <typename E, int C, int VPT>
int run_loss_vpt(const void *Pz, const void *Plab, void *Pdz, float *loss, float *stats, const Geo &g, float w_dice,
             float w_ce, float eps, void *ws, hipStream_t s) {
    const LossGeo l = make_loss_geo(g);
    const unsigned nblk = (l.nvox + kChunk - 1) / kChunk;
    float *part = static_cast<float *>(ws);
    float *st = stats ? stats : part + static_cast<size_t>(nblk) * (3 * C + 1);
    hipLaunchKernelGGL((loss_stats_kernel<E, C, VPT>), dim3(nblk), dim3(kThreads), 0, s, static_cast<const E *>(Pz),
                       static_cast<const E *>(Plab), part, l);
    int rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    rc = launch_reduce_partials(part, st, static_cast<int>(nblk), 3 * C + 1, s);
    if (rc != SP_OK) return rc;
    const unsigned gblk = Pdz ? (l.nvox / VPT + kThreads - 1) / kThreads : 1;
    hipLaunchKernelGGL((loss_grad_kernel<E, C, VPT>), dim3(gblk), dim3(kThreads), 0, s, static_cast<const E *>(Pz),
                       static_cast<const E *>(Plab), st, static_cast<E *>(Pdz), loss, l, w_dice, w_ce, eps);
    return record_hip(hipGetLastError());
}

template <typename E, int C>
int run_loss(const void *Pz, const void *Plab, void *Pdz, float *loss, float *stats, const Geo &g, float w_dice,
             float w_ce, float eps, void *ws, hipStream_t s) {
    if (g.tw % 8 == 0) return run_loss_vpt<E, C, 8>(Pz, Plab, Pdz, loss, stats, g, w_dice, w_ce, eps, ws, s);
    return run_loss_vpt<E, C, 1>(Pz, Plab, Pdz, loss, stats, g, w_dice, w_ce, eps, ws, s);
}

}  // namespace

bool loss_supported(const Geo &g, int classes) {
    return classes >= 2 && classes <= 4 && 1LL * g.ntiles * g.int_vox <= 0xffffff00LL;
}

size_t loss_ws_bytes(const Geo &g, int classes) {
    const size_t nblk = (static_cast<size_t>(g.ntiles) * g.int_vox + kChunk - 1) / kChunk;
    return (nblk + 1) * (3 * classes + 1) * sizeof(float);
}

int launch_loss(const void *Pz, const void *Plab, void *Pdz, float *loss, float *stats, const Geo &g, int classes,
                sp_dtype_t dt, float w_dice, float w_ce, float eps, void *ws, hipStream_t s) {
#define SP3D_LOSS(E)                                                                                         \
    switch (classes) {                                                                                       \
    case 2: return run_loss<E, 2>(Pz, Plab, Pdz, loss, stats, g, w_dice, w_ce, eps, ws, s);                  \
    case 3: return run_loss<E, 3>(Pz, Plab, Pdz, loss, stats, g, w_dice, w_ce, eps, ws, s);                  \
    default: return run_loss<E, 4>(Pz, Plab, Pdz, loss, stats, g, w_dice, w_ce, eps, ws, s);                 \
    }
    if (dt == SP_BF16) { SP3D_LOSS(uint16_t) }
    SP3D_LOSS(float)
#undef SP3D_LOSS
}

}  // namespace sp3d
