// Bandwidth-bound data movement kernels: volume <-> padded tiles, halo pack / unpack, ReLU mask.
// All copies are bit-exact; addresses are computed per contiguous run so that global accesses
// are as wide as the voxel record (C * element size) allows, up to 16 bytes per lane.
#include "common.h"

namespace sp3d {

namespace {

constexpr int kThreads = 256;

// widest power-of-two vector (bytes, <= 16) that divides the voxel record size
int vec_bytes(size_t rec) {
    int v = 16;
    while (rec % v) v >>= 1;
    return v;
}

template <int B> struct VecT;
template <> struct VecT<2> { using type = uint16_t; };
template <> struct VecT<4> { using type = uint32_t; };
template <> struct VecT<8> { using type = uint2; };
template <> struct VecT<16> { using type = uint4; };

template <typename T> __device__ __forceinline__ T zero_vec();
template <> __device__ __forceinline__ uint16_t zero_vec<uint16_t>() { return 0; }
template <> __device__ __forceinline__ uint32_t zero_vec<uint32_t>() { return 0; }
template <> __device__ __forceinline__ uint2 zero_vec<uint2>() { return make_uint2(0, 0); }
template <> __device__ __forceinline__ uint4 zero_vec<uint4>() { return make_uint4(0, 0, 0, 0); }

// ---------------------------------------------------------------------------------------------
// partition / unpartition.  A "row" is the run of tw voxels of one tile at fixed (ld, lh); it is
// contiguous both in the volume and in the padded tile.  tpr threads serve one row.
struct PartArgs {
    Geo g;
    int rowvecs;       // vectors per row
    int tpr;           // threads per row (power of two, <= 256)
    long long rows;    // ntiles * td * th
    int vpv_num;       // vectors per voxel numerator: rec / vec  (rows are addressed in vectors)
};

template <typename T, bool INVERSE>
__global__ __launch_bounds__(kThreads) void partition_kernel(const T *__restrict__ src,
                                                             T *__restrict__ dst, PartArgs a) {
    const Geo &g = a.g;
    const int rpb = kThreads / a.tpr;
    const long long row = 1LL * blockIdx.x * rpb + threadIdx.x / a.tpr;
    if (row >= a.rows) return;
    const int lane = threadIdx.x % a.tpr;
    // row -> (tile, ld, lh)
    const unsigned rows_per_tile = static_cast<unsigned>(g.td) * g.th;
    const unsigned tile = static_cast<unsigned>(row / rows_per_tile);
    const unsigned r = static_cast<unsigned>(row % rows_per_tile);
    const unsigned ld = r / g.th, lh = r % g.th;
    // tile -> (n, a, b, c)
    const unsigned tc = tile % g.gw, tb = (tile / g.gw) % g.gh;
    const unsigned ta = (tile / (g.gw * g.gh)) % g.gd, tn = tile / (g.gw * g.gh * g.gd);
    const long long D = 1LL * g.gd * g.td, H = 1LL * g.gh * g.th, W = 1LL * g.gw * g.tw;
    const long long vvox = ((tn * D + ta * g.td + ld) * H + tb * g.th + lh) * W + 1LL * tc * g.tw;
    const long long pvox = tile * g.tile_vox +
                           (1LL * (ld + g.halo) * g.ph + lh + g.halo) * g.pw + g.halo;
    const T *v = (INVERSE ? dst : src) + vvox * a.vpv_num;   // volume side
    const T *p = (INVERSE ? src : dst) + pvox * a.vpv_num;   // padded side
    if (INVERSE) {
        T *out = const_cast<T *>(v);
        for (int j = lane; j < a.rowvecs; j += a.tpr) out[j] = p[j];
    } else {
        T *out = const_cast<T *>(p);
        for (int j = lane; j < a.rowvecs; j += a.tpr) out[j] = v[j];
    }
}

template <int VB>
int partition_dispatch(const void *vol, void *P, const PartArgs &a, bool inverse, hipStream_t s) {
    using T = typename VecT<VB>::type;
    const int rpb = kThreads / a.tpr;
    const long long blocks = (a.rows + rpb - 1) / rpb;
    if (blocks > 0x7fffffffLL) return SP_EGEOM;
    dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    if (inverse)
        hipLaunchKernelGGL((partition_kernel<T, true>), grid, block, 0, s,
                           static_cast<const T *>(P), static_cast<T *>(const_cast<void *>(vol)), a);
    else
        hipLaunchKernelGGL((partition_kernel<T, false>), grid, block, 0, s,
                           static_cast<const T *>(vol), static_cast<T *>(P), a);
    return record_hip(hipGetLastError());
}

// ---------------------------------------------------------------------------------------------
// halo pack / unpack.  One block serves a chunk of one region of one tile.
constexpr int kHaloUnroll = 4;
constexpr int kHaloChunk = kThreads * kHaloUnroll;   // vectors per block

struct HaloArgs {
    Geo g;
    RegionTable t;
    int blk_prefix[27];   // first block (within a tile) of each region; [26] = blocks per tile
    int vpv;              // vectors per voxel
};

template <typename T, bool UNPACK>
__global__ __launch_bounds__(kThreads) void halo_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                        HaloArgs a) {
    const Geo &g = a.g;
    const unsigned bpt = a.blk_prefix[26];
    const unsigned tile = blockIdx.x / bpt, rem = blockIdx.x % bpt;
    int ri = 0;
    while (ri < 25 && static_cast<unsigned>(a.blk_prefix[ri + 1]) <= rem) ++ri;   // uniform
    const Region &r = a.t.r[ri];
    const unsigned chunk = rem - a.blk_prefix[ri];
    const unsigned nvec = static_cast<unsigned>(r.ext[0]) * r.ext[1] * r.ext[2] * a.vpv;

    long long nb_msg = -1;   // UNPACK: voxel offset of the neighbour's message region, -1 = none
    if (UNPACK) {
        const int tc = tile % g.gw, tb = (tile / g.gw) % g.gh;
        const int ta = (tile / (g.gw * g.gh)) % g.gd, tn = tile / (g.gw * g.gh * g.gd);
        const int na = ta + r.delta[0], nb = tb + r.delta[1], nc = tc + r.delta[2];
        if (na >= 0 && na < g.gd && nb >= 0 && nb < g.gh && nc >= 0 && nc < g.gw) {
            const long long ntile = ((1LL * tn * g.gd + na) * g.gh + nb) * g.gw + nc;
            nb_msg = ntile * g.msg_vox + a.t.r[r.opposite].off;
        }
    }
    const int *org = UNPACK ? r.recv : r.send;
    const long long pbase = tile * g.tile_vox;
    const long long mbase = tile * g.msg_vox + r.off;
    const unsigned ehw = static_cast<unsigned>(r.ext[1]) * r.ext[2];
#pragma unroll
    for (int u = 0; u < kHaloUnroll; ++u) {
        const unsigned j = chunk * kHaloChunk + u * kThreads + threadIdx.x;
        if (j >= nvec) break;
        const unsigned vox = j / a.vpv, cv = j % a.vpv;
        const unsigned ld = vox / ehw, q = vox % ehw;
        const unsigned lh = q / r.ext[2], lw = q % r.ext[2];
        const long long pvox = pbase + (1LL * (org[0] + ld) * g.ph + org[1] + lh) * g.pw + org[2] + lw;
        if (UNPACK) {
            T v = zero_vec<T>();
            if (nb_msg >= 0) v = src[(nb_msg + vox) * a.vpv + cv];
            dst[pvox * a.vpv + cv] = v;
        } else {
            dst[(mbase + vox) * a.vpv + cv] = src[pvox * a.vpv + cv];
        }
    }
}

template <int VB>
int halo_dispatch(const void *src, void *dst, HaloArgs &a, bool unpack, hipStream_t s) {
    using T = typename VecT<VB>::type;
    int acc = 0;
    for (int i = 0; i < 26; ++i) {
        a.blk_prefix[i] = acc;
        const long long nvec = 1LL * a.t.r[i].ext[0] * a.t.r[i].ext[1] * a.t.r[i].ext[2] * a.vpv;
        if (nvec > 0xffffffffLL) return SP_EGEOM;
        acc += static_cast<int>((nvec + kHaloChunk - 1) / kHaloChunk);
    }
    a.blk_prefix[26] = acc;
    const long long blocks = 1LL * acc * a.g.ntiles;
    if (blocks > 0x7fffffffLL) return SP_EGEOM;
    dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    if (unpack)
        hipLaunchKernelGGL((halo_kernel<T, true>), grid, block, 0, s, static_cast<const T *>(src),
                           static_cast<T *>(dst), a);
    else
        hipLaunchKernelGGL((halo_kernel<T, false>), grid, block, 0, s, static_cast<const T *>(src),
                           static_cast<T *>(dst), a);
    return record_hip(hipGetLastError());
}

// ---------------------------------------------------------------------------------------------
// ReLU backward mask: dz = dy where y > 0 else 0.
template <typename E> __device__ __forceinline__ bool positive(E v);
template <> __device__ __forceinline__ bool positive<float>(float v) { return v > 0.f; }
// bf16 bits: positive and non-zero (NaN counts as not positive only if its sign bit is set)
template <> __device__ __forceinline__ bool positive<uint16_t>(uint16_t v) {
    return (v & 0x8000u) == 0 && (v & 0x7fffu) != 0 && (v & 0x7fffu) <= 0x7f80u;
}

template <typename E>
__global__ __launch_bounds__(kThreads) void relu_bwd_kernel(const E *__restrict__ dy,
                                                            const E *__restrict__ y,
                                                            E *__restrict__ dz, size_t n) {
    const size_t stride = static_cast<size_t>(gridDim.x) * kThreads;
    for (size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x; i < n; i += stride)
        dz[i] = positive<E>(y[i]) ? dy[i] : E(0);
}

}  // namespace

int launch_partition(const void *vol, void *P, const Geo &g, int c, sp_dtype_t dt, bool inverse,
                     hipStream_t s) {
    const size_t rec = static_cast<size_t>(c) * elem_size(dt);
    const int vb = vec_bytes(rec);
    PartArgs a;
    a.g = g;
    a.vpv_num = static_cast<int>(rec / vb);
    const long long rowvecs = 1LL * g.tw * a.vpv_num;
    if (rowvecs > 0x7fffffffLL) return SP_EGEOM;
    a.rowvecs = static_cast<int>(rowvecs);
    int tpr = 1;
    while (tpr < kThreads && tpr < a.rowvecs) tpr <<= 1;
    a.tpr = tpr;
    a.rows = 1LL * g.ntiles * g.td * g.th;
    switch (vb) {
    case 16: return partition_dispatch<16>(vol, P, a, inverse, s);
    case 8: return partition_dispatch<8>(vol, P, a, inverse, s);
    case 4: return partition_dispatch<4>(vol, P, a, inverse, s);
    default: return partition_dispatch<2>(vol, P, a, inverse, s);
    }
}

static int halo_launch(const void *src, void *dst, const Geo &g, int c, sp_dtype_t dt, bool unpack,
                       hipStream_t s) {
    const size_t rec = static_cast<size_t>(c) * elem_size(dt);
    const int vb = vec_bytes(rec);
    HaloArgs a;
    a.g = g;
    make_regions(g, &a.t);
    a.vpv = static_cast<int>(rec / vb);
    switch (vb) {
    case 16: return halo_dispatch<16>(src, dst, a, unpack, s);
    case 8: return halo_dispatch<8>(src, dst, a, unpack, s);
    case 4: return halo_dispatch<4>(src, dst, a, unpack, s);
    default: return halo_dispatch<2>(src, dst, a, unpack, s);
    }
}

int launch_halo_pack(const void *P, void *msg, const Geo &g, int c, sp_dtype_t dt, hipStream_t s) {
    return halo_launch(P, msg, g, c, dt, false, s);
}

int launch_halo_unpack(void *P, const void *msg, const Geo &g, int c, sp_dtype_t dt, hipStream_t s) {
    return halo_launch(msg, P, g, c, dt, true, s);
}

int launch_relu_bwd(const void *dy, const void *y, void *dz, size_t elems, sp_dtype_t dt,
                    hipStream_t s) {
    if (elems == 0) return SP_OK;
    size_t blocks = (elems + kThreads - 1) / kThreads;
    if (blocks > 65536) blocks = 65536;
    dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    if (dt == SP_BF16)
        hipLaunchKernelGGL(relu_bwd_kernel<uint16_t>, grid, block, 0, s,
                           static_cast<const uint16_t *>(dy), static_cast<const uint16_t *>(y),
                           static_cast<uint16_t *>(dz), elems);
    else
        hipLaunchKernelGGL(relu_bwd_kernel<float>, grid, block, 0, s, static_cast<const float *>(dy),
                           static_cast<const float *>(y), static_cast<float *>(dz), elems);
    return record_hip(hipGetLastError());
}

}  // namespace sp3d
