// Bandwidth-bound data movement kernels: volume <-> padded tiles, halo pack / unpack, ReLU mask.
// All copies are bit-exact; addresses are computed per contiguous run so that global accesses
// are as wide as the voxel record (C * element size) allows, up to 16 bytes per lane.
#include "common.h"

#include <algorithm>

namespace sp3d {

namespace {

constexpr int kThreads = 256;

// widest power-of-two vector (bytes, <= 16) that divides the voxel record size
int vec_bytes(size_t rec) {
    int v = 16;
    while (rec % v) v >>= 1;
    return v;
}

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
template <int B> struct VecT;
template <> struct VecT<2> { using type = uint16_t; };
template <> struct VecT<4> { using type = uint32_t; };
template <> struct VecT<8> { using type = u32x2; };
template <> struct VecT<16> { using type = u32x4; };

// 16 bytes at an address that is only aligned to the element (2 or 4 bytes): rows of voxel records whose size
// does not divide 16 (3 channels of bf16 = 6 bytes) are still contiguous runs of bytes, and the hardware
// serves wide accesses at any alignment
struct __attribute__((packed, aligned(2))) Bytes16 { uint32_t w[4]; };

template <typename T> __device__ __forceinline__ T zero_vec() { return T(0); }

// Streaming accesses: every byte is touched exactly once, so bypass-friendly (non-temporal) loads and
// stores are used; measured copy ceiling on MI355X: 6.5 TB/s against 6.1 TB/s with plain accesses.
template <typename T> __device__ __forceinline__ T ld_stream(const T *p) { return __builtin_nontemporal_load(p); }
template <typename T> __device__ __forceinline__ void st_stream(T *p, T v) { __builtin_nontemporal_store(v, p); }
template <> __device__ __forceinline__ Bytes16 ld_stream<Bytes16>(const Bytes16 *p) { return *p; }
template <> __device__ __forceinline__ void st_stream<Bytes16>(Bytes16 *p, Bytes16 v) { *p = v; }

// Workgroups are dealt to the 8 XCDs of the chip round-robin (workgroup i runs on XCD i % 8).  With block i working
// on the i-th piece of memory, every XCD - each with its own L2 - touches every eighth 4 KB piece; with the
// remapping below each XCD streams through one contiguous eighth of the blocks instead.  For the copies into and
// out of padded tiles that is the difference between 5.8 and 6.6 TB/s (the rate of a plain linear copy); a linear
// copy does not care.  Grids are rounded up to a multiple of 8; ids past the last block do nothing.
__device__ __forceinline__ unsigned xcd_contiguous_block() {
    return (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
}
inline unsigned round_up8(unsigned blocks) { return (blocks + 7u) / 8u * 8u; }

// ---------------------------------------------------------------------------------------------
// partition / unpartition.  A "row" is the run of tw voxels of one tile at fixed (ld, lh); it is
// contiguous both in the volume and in the padded tile.  Many small workgroups stream
// best on this chip; a block covers kVpt chunks of 256 vectors of a row (or of several short rows).
struct PartArgs {
    Geo g;
    int rowvecs;       // vectors per row
    int tpr;           // threads per row chunk (power of two, <= 256)
    unsigned nchunks;  // rows * cpr (row chunks in total; checked to fit 32 bits)
    int vpv_num;       // vectors per voxel: rec / vec  (rows are addressed in vectors); Bytes16 rows: bytes per voxel
    FastDiv cpr;       // chunks of tpr vectors per row
    FastDiv rows_per_tile, th, gw, gh, gd;
};

// Vectors per thread in the halo kernels below: the loads of all of them are issued before the first store,
// which keeps more bytes in flight per wave (two measured best; one or four are slower).
constexpr int kVpt = 2;

template <typename T> __device__ __forceinline__ T *at(T *p, long long off) { return p + off; }
template <> __device__ __forceinline__ const Bytes16 *at<const Bytes16>(const Bytes16 *p, long long off) {
    return reinterpret_cast<const Bytes16 *>(reinterpret_cast<const char *>(p) + off);
}
template <> __device__ __forceinline__ Bytes16 *at<Bytes16>(Bytes16 *p, long long off) {
    return reinterpret_cast<Bytes16 *>(reinterpret_cast<char *>(p) + off);
}

// Offsets (source, destination) of vector j of row chunk rc, and whether it exists.  With rc taken from the
// block index alone the whole row / tile decode is wave-uniform and runs on the scalar unit.
template <typename T, bool INVERSE>
__device__ __forceinline__ bool partition_offsets(const PartArgs &a, unsigned rc, unsigned jl, long long *so,
                                                  long long *dof) {
    const Geo &g = a.g;
    const long long D = 1LL * g.gd * g.td, H = 1LL * g.gh * g.th, W = 1LL * g.gw * g.tw;
    const unsigned rcc = rc < a.nchunks ? rc : 0;
    const unsigned row = fdiv(rcc, a.cpr);
    const unsigned j = fmod_(rcc, row, a.cpr) * a.tpr + jl;
    // row -> (tile, ld, lh)
    const unsigned tile = fdiv(row, a.rows_per_tile);
    const unsigned r = fmod_(row, tile, a.rows_per_tile);
    const unsigned ld = fdiv(r, a.th), lh = fmod_(r, ld, a.th);
    // tile -> (n, a, b, c)
    const unsigned t1 = fdiv(tile, a.gw), tc = fmod_(tile, t1, a.gw);
    const unsigned t2 = fdiv(t1, a.gh), tb = fmod_(t1, t2, a.gh);
    const unsigned tn = fdiv(t2, a.gd), ta = fmod_(t2, tn, a.gd);
    const long long vvox = ((tn * D + ta * g.td + ld) * H + tb * g.th + lh) * W + 1LL * tc * g.tw;
    const long long pvox = tile * g.tile_vox + (1LL * (ld + g.halo) * g.ph + lh + g.halo) * g.pw + g.halo;
    // offsets in vectors; rows of Bytes16 start at any even byte, so those are kept in bytes
    constexpr long long JS = std::is_same<T, Bytes16>::value ? 16 : 1;
    *so = (INVERSE ? pvox : vvox) * a.vpv_num + j * JS;
    *dof = (INVERSE ? vvox : pvox) * a.vpv_num + j * JS;
    return rc < a.nchunks && j < static_cast<unsigned>(a.rowvecs);
}

template <typename T, bool INVERSE, int VPT>
__global__ __launch_bounds__(kThreads) void partition_kernel(const T *__restrict__ src,
                                                             T *__restrict__ dst, PartArgs a) {
    T v[VPT];
    long long so[VPT], do_[VPT];
    bool ok[VPT];
    const unsigned bid = xcd_contiguous_block();   // blocks past the last chunk find ok[] false below
    if (a.tpr == kThreads) {   // a block per row chunk (rows of at least 256 vectors): uniform decode
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            ok[k] = partition_offsets<T, INVERSE>(a, bid * VPT + k, threadIdx.x, &so[k], &do_[k]);
            if (ok[k]) v[k] = ld_stream(at(src, so[k]));
        }
    } else {
        const unsigned rpb = kThreads / a.tpr;                  // row chunks per block and pass
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            ok[k] = partition_offsets<T, INVERSE>(a, (bid * VPT + k) * rpb + threadIdx.x / a.tpr,
                                                  threadIdx.x % a.tpr, &so[k], &do_[k]);
            if (ok[k]) v[k] = ld_stream(at(src, so[k]));
        }
    }
#pragma unroll
    for (int k = 0; k < VPT; ++k)
        if (ok[k]) st_stream(at(dst, do_[k]), v[k]);
}

template <typename T>
int partition_dispatch(const void *vol, void *P, const PartArgs &a, bool inverse, hipStream_t s) {
    // one vector per thread in both directions: with the XCD-contiguous block order two were slower (before it,
    // gathering from the padded tiles gained from two)
    const unsigned rpb = kThreads / a.tpr;
    const unsigned blocks = round_up8((a.nchunks + rpb - 1) / rpb);
    dim3 grid(blocks), block(kThreads);
    if (inverse)
        hipLaunchKernelGGL((partition_kernel<T, true, 1>), grid, block, 0, s,
                           static_cast<const T *>(P), static_cast<T *>(const_cast<void *>(vol)), a);
    else
        hipLaunchKernelGGL((partition_kernel<T, false, 1>), grid, block, 0, s,
                           static_cast<const T *>(vol), static_cast<T *>(P), a);
    return record_hip(hipGetLastError());
}

// ---------------------------------------------------------------------------------------------
// halo pack / unpack.  One block serves a chunk of one region of one tile; a block whose region the call leaves
// alone (SP_HALO_*: the tile has no neighbour in that direction) returns at once.
constexpr int kHaloChunk = kThreads * kVpt;   // vectors per block

// Everything a block needs to know about its region, in one 112-byte record: after the search for the block's
// region the scalar unit fetches it with a single load (the region table, its opposite entry, the per-region
// dividers and the order table were four dependent loads before; a wave spends more of its life on this preamble
// than on its two memory round trips).  Records are in the order the regions' blocks follow each other inside a
// tile: largest first, so that the search ends after a step or two for nearly every block (the message layout
// is not affected: it is given by the regions' offsets).
struct HaloRec {
    int ext[3];           // extents (d,h,w) of the region
    int org[3];           // pack: origin of the sent box; unpack / exchange: origin of the margin box (padded coordinates)
    int delta[3];         // direction
    int nsend[3];         // exchange: origin of the box the neighbour would have packed (the opposite region's)
    long long off;        // voxel offset of the region inside a tile's message
    long long off_opp;    // ... of the opposite region (what unpack reads from the neighbour's message)
    FastDiv ehw, ew;      // ext[1]*ext[2] and ext[2]
    unsigned nvec;        // vectors of the region
    unsigned nch;         // its blocks
    int whole_rows;       // 1: a row is a whole multiple of a block's vectors
    int pad;
};
static_assert(sizeof(HaloRec) == 112, "one record = two scalar loads");

struct HaloArgs {
    Geo g;
    HaloRec rec[26];
    int blk_prefix[27];   // first block (within a tile) of the region at each position; [26] = blocks per tile
    FastDiv vpv;          // vectors per voxel
    FastDiv bpt, gw, gh, gd;
    int skip;             // 1: regions whose direction leads outside the grid are left alone (SP_HALO_*)
};
static_assert(sizeof(HaloArgs) + 16 <= 4096, "kernel arguments");

// MODE: kPack = tile interiors -> messages; kUnpack = neighbours' messages -> margins (zeros where the
// neighbour is outside the grid); kExchange = both at once when all tiles share one memory: every margin
// region is read straight from the neighbour's interior (src and dst are then the same tensor; the
// reads touch interiors only and the writes margins only).
enum HaloMode { kPack = 0, kUnpack = 1, kExchange = 2 };

template <typename T, int MODE>
__global__ __launch_bounds__(kThreads) void halo_kernel(const T *src, T *dst, HaloArgs a) {
    constexpr bool UNPACK = MODE != kPack;
    const Geo &g = a.g;
    const unsigned tile = fdiv(blockIdx.x, a.bpt), rem = fmod_(blockIdx.x, tile, a.bpt);
    int pi = 0;
    while (pi < 25 && static_cast<unsigned>(a.blk_prefix[pi + 1]) <= rem) ++pi;   // uniform
    const HaloRec &r = a.rec[pi];
    unsigned chunk = rem - a.blk_prefix[pi];
    const unsigned nvec = r.nvec;
    if (chunk * kHaloChunk >= nvec) return;   // uniform; cannot happen with the block counts of halo_dispatch

    long long nb_msg = -1;   // UNPACK: voxel offset of the neighbour's message region, -1 = none
    if (UNPACK || a.skip) {
        const unsigned t1 = fdiv(tile, a.gw), tc = fmod_(tile, t1, a.gw);
        const unsigned t2 = fdiv(t1, a.gh), tb = fmod_(t1, t2, a.gh);
        const unsigned tn = fdiv(t2, a.gd), ta = fmod_(t2, tn, a.gd);
        const int na = static_cast<int>(ta) + r.delta[0], nb = static_cast<int>(tb) + r.delta[1];
        const int nc = static_cast<int>(tc) + r.delta[2];
        if (na >= 0 && na < g.gd && nb >= 0 && nb < g.gh && nc >= 0 && nc < g.gw) {
            const long long ntile = ((1LL * tn * g.gd + na) * g.gh + nb) * g.gw + nc;
            nb_msg = MODE == kExchange ? ntile : ntile * g.msg_vox + r.off_opp;
        } else if (a.skip) {
            return;          // uniform: nobody receives this region / its margin holds zeros already
        }
    }
    // Consecutive blocks run on consecutive XCDs.  In a region of many chunks every XCD gets a contiguous
    // eighth of the chunks instead of every eighth chunk (as in xcd_contiguous_block(), but per tile and region:
    // over the whole grid the XCDs would get unequal shares of the zero-fill work).  A bijection of the chunks.
    {
        const unsigned nch = r.nch;
        if (nch >= 64 && (nch & 7u) == 0) chunk = (chunk & 7u) * (nch >> 3) + (chunk >> 3);
    }
    const long long msg0 = UNPACK ? nb_msg : tile * g.msg_vox + r.off;   // message region of this block
    T v[kVpt];
    long long mo[kVpt], po[kVpt];   // vector offsets in the message and in the padded tensor
    bool ok[kVpt];
    // vector j of the region -> its offsets in the padded tensor and in the message (or, kExchange, in the
    // neighbour's interior)
    auto locate = [&](unsigned j, long long *pout, long long *mout) {
        const unsigned vox = fdiv(j, a.vpv), cv = fmod_(j, vox, a.vpv);
        const unsigned ld = fdiv(vox, r.ehw), q = fmod_(vox, ld, r.ehw);
        const unsigned lh = fdiv(q, r.ew), lw = fmod_(q, lh, r.ew);
        const long long pvox = tile * g.tile_vox + (1LL * (r.org[0] + ld) * g.ph + r.org[1] + lh) * g.pw + r.org[2] + lw;
        *pout = pvox * a.vpv.d + cv;
        if (MODE == kExchange)
            *mout = (nb_msg * g.tile_vox + (1LL * (r.nsend[0] + ld) * g.ph + r.nsend[1] + lh) * g.pw + r.nsend[2] + lw) *
                        a.vpv.d + cv;
        else
            *mout = (msg0 + vox) * a.vpv.d + cv;
    };
    if (r.whole_rows) {
        // rows that are whole multiples of a block's vectors (the D and H faces of large tiles): the block lies
        // inside one row, so its first vector is located once, on the scalar unit, and a lane only adds its index
        long long p0, m0;
        locate(chunk * kHaloChunk, &p0, &m0);
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            ok[k] = true;
            po[k] = p0 + k * kThreads + threadIdx.x;
            mo[k] = m0 + k * kThreads + threadIdx.x;
        }
    } else {
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            const unsigned j = chunk * kHaloChunk + k * kThreads + threadIdx.x;
            ok[k] = j < nvec;
            locate(ok[k] ? j : 0, &po[k], &mo[k]);
        }
    }
#pragma unroll
    for (int k = 0; k < kVpt; ++k) {
        v[k] = zero_vec<T>();
        if (ok[k] && (!UNPACK || nb_msg >= 0)) v[k] = ld_stream(src + (UNPACK ? mo[k] : po[k]));
    }
#pragma unroll
    for (int k = 0; k < kVpt; ++k)
        if (ok[k]) st_stream(dst + (UNPACK ? po[k] : mo[k]), v[k]);
}

template <int VB>
int halo_dispatch(const void *src, void *dst, HaloArgs &a, const RegionTable &t, int mode, hipStream_t s) {
    using T = typename VecT<VB>::type;
    int nblk[26], order[26];
    long long nvecs[26];
    for (int i = 0; i < 26; ++i) {
        const long long nvec = 1LL * t.r[i].ext[0] * t.r[i].ext[1] * t.r[i].ext[2] * a.vpv.d;
        if (nvec > 0xffffff00LL) return SP_EGEOM;
        nvecs[i] = nvec;
        // 2-D variant: slices do not interact, the regions above and below a tile are not moved
        nblk[i] = (a.g.flat && t.r[i].delta[0] != 0) ? 0 : static_cast<int>((nvec + kHaloChunk - 1) / kHaloChunk);
        // a direction along an axis that the grid does not split leads outside the grid for every tile: with
        // SP_HALO_* such a region gets no blocks at all (instead of blocks that find that out and return)
        const int gdim[3] = {a.g.gd, a.g.gh, a.g.gw};
        for (int k = 0; k < 3; ++k)
            if (a.skip && t.r[i].delta[k] != 0 && gdim[k] == 1) nblk[i] = 0;
        order[i] = i;
    }
    std::stable_sort(order, order + 26, [&](int x, int y) { return nblk[x] > nblk[y]; });
    int acc = 0;
    for (int p = 0; p < 26; ++p) {
        const Region &r = t.r[order[p]], &o = t.r[r.opposite];
        HaloRec &h = a.rec[p];
        for (int k = 0; k < 3; ++k) {
            h.ext[k] = r.ext[k];
            h.org[k] = mode == kPack ? r.send[k] : r.recv[k];
            h.delta[k] = r.delta[k];
            h.nsend[k] = o.send[k];
        }
        h.off = r.off;
        h.off_opp = o.off;
        h.ehw = make_fastdiv(static_cast<uint32_t>(r.ext[1]) * r.ext[2]);
        h.ew = make_fastdiv(r.ext[2]);
        h.nvec = static_cast<unsigned>(nvecs[order[p]]);
        h.nch = static_cast<unsigned>(nblk[order[p]]);
        h.whole_rows = (static_cast<unsigned>(r.ext[2]) * a.vpv.d) % kHaloChunk == 0 ? 1 : 0;
        h.pad = 0;
        a.blk_prefix[p] = acc;
        acc += nblk[order[p]];
    }
    a.blk_prefix[26] = acc;
    if (acc == 0) return SP_OK;       // one tile and nothing to do beyond the volume border: no launch
    a.bpt = make_fastdiv(acc);
    a.gw = make_fastdiv(a.g.gw);
    a.gh = make_fastdiv(a.g.gh);
    a.gd = make_fastdiv(a.g.gd);
    const long long blocks = 1LL * acc * a.g.ntiles;
    if (blocks > 0x7fffffffLL) return SP_EGEOM;
    dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    if (mode == kUnpack)
        hipLaunchKernelGGL((halo_kernel<T, kUnpack>), grid, block, 0, s, static_cast<const T *>(src),
                           static_cast<T *>(dst), a);
    else if (mode == kExchange)
        hipLaunchKernelGGL((halo_kernel<T, kExchange>), grid, block, 0, s, static_cast<const T *>(src),
                           static_cast<T *>(dst), a);
    else
        hipLaunchKernelGGL((halo_kernel<T, kPack>), grid, block, 0, s, static_cast<const T *>(src),
                           static_cast<T *>(dst), a);
    return record_hip(hipGetLastError());
}

// ---------------------------------------------------------------------------------------------
// ReLU backward mask: dz = dy where y > 0 else 0.
template <typename E> __device__ __forceinline__ bool positive(E v);
template <> __device__ __forceinline__ bool positive<float>(float v) { return v > 0.f; }
// bf16 bits: positive, non-zero and not NaN (a NaN of either sign is not positive)
template <> __device__ __forceinline__ bool positive<uint16_t>(uint16_t v) {
    return (v & 0x8000u) == 0 && (v & 0x7fffu) != 0 && (v & 0x7fffu) <= 0x7f80u;
}

// (dz may be the same tensor as dy, so no __restrict__ on those two: every thread reads and writes its own index)
template <typename E>
__global__ __launch_bounds__(kThreads) void relu_bwd_kernel(const E *dy, const E *__restrict__ y, E *dz, size_t n) {
    const size_t stride = static_cast<size_t>(gridDim.x) * kThreads;
    for (size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x; i < n; i += stride)
        dz[i] = positive<E>(y[i]) ? dy[i] : E(0);
}

// 16-byte variant for bf16 (8 elements per thread): mask built from the sign/zero test of each half word
__global__ __launch_bounds__(kThreads) void relu_bwd_bf16x8_kernel(const u32x4 *dy, const u32x4 *__restrict__ y,
                                                                   u32x4 *dz, size_t nvec) {
    const size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i >= nvec) return;
    const u32x4 g = dy[i], v = y[i];
    u32x4 o;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t lo = positive<uint16_t>(static_cast<uint16_t>(v[k] & 0xffffu)) ? 0x0000ffffu : 0u;
        const uint32_t hi = positive<uint16_t>(static_cast<uint16_t>(v[k] >> 16)) ? 0xffff0000u : 0u;
        o[k] = g[k] & (lo | hi);
    }
    st_stream(&dz[i], o);
}

}  // namespace

int launch_partition(const void *vol, void *P, const Geo &g, int c, sp_dtype_t dt, bool inverse,
                     hipStream_t s) {
    const size_t rec = static_cast<size_t>(c) * elem_size(dt);
    int vb = vec_bytes(rec);
    // narrow records whose rows are still whole multiples of 16 bytes: copy the rows as bytes, 16 at a time
    const bool as_bytes = vb < 16 && (static_cast<size_t>(g.tw) * rec) % 16 == 0;
    if (as_bytes) vb = 16;
    PartArgs a;
    a.g = g;
    a.vpv_num = as_bytes ? static_cast<int>(rec) : static_cast<int>(rec / vb);
    const long long rowvecs = as_bytes ? static_cast<long long>(g.tw * rec / 16) : 1LL * g.tw * a.vpv_num;
    if (rowvecs > 0x7fffffffLL) return SP_EGEOM;
    a.rowvecs = static_cast<int>(rowvecs);
    int tpr = 1;
    while (tpr < kThreads && tpr < a.rowvecs) tpr <<= 1;
    a.tpr = tpr;
    const long long cpr = (a.rowvecs + tpr - 1) / tpr;
    const long long nchunks = 1LL * g.ntiles * g.td * g.th * cpr;
    if (nchunks > 0xffffe000LL) return SP_EGEOM;   // room for the rounding up to whole blocks and to 8 blocks
    a.nchunks = static_cast<unsigned>(nchunks);
    a.cpr = make_fastdiv(static_cast<uint32_t>(cpr));
    a.rows_per_tile = make_fastdiv(static_cast<uint32_t>(g.td) * g.th);
    a.th = make_fastdiv(g.th);
    a.gw = make_fastdiv(g.gw);
    a.gh = make_fastdiv(g.gh);
    a.gd = make_fastdiv(g.gd);
    if (as_bytes) return partition_dispatch<Bytes16>(vol, P, a, inverse, s);
    switch (vb) {
    case 16: return partition_dispatch<VecT<16>::type>(vol, P, a, inverse, s);
    case 8: return partition_dispatch<VecT<8>::type>(vol, P, a, inverse, s);
    case 4: return partition_dispatch<VecT<4>::type>(vol, P, a, inverse, s);
    default: return partition_dispatch<VecT<2>::type>(vol, P, a, inverse, s);
    }
}

static int halo_launch(const void *src, void *dst, const Geo &g, int c, sp_dtype_t dt, int mode, int border,
                       hipStream_t s) {
    const size_t rec = static_cast<size_t>(c) * elem_size(dt);
    const int vb = vec_bytes(rec);
    HaloArgs a;
    a.g = g;
    a.skip = (border & (mode == kPack ? SP_HALO_SKIP_SEND : SP_HALO_KEEP_ZERO)) ? 1 : 0;
    RegionTable t;
    make_regions(g, &t);
    a.vpv = make_fastdiv(static_cast<uint32_t>(rec / vb));
    switch (vb) {
    case 16: return halo_dispatch<16>(src, dst, a, t, mode, s);
    case 8: return halo_dispatch<8>(src, dst, a, t, mode, s);
    case 4: return halo_dispatch<4>(src, dst, a, t, mode, s);
    default: return halo_dispatch<2>(src, dst, a, t, mode, s);
    }
}

int launch_halo_pack(const void *P, void *msg, const Geo &g, int c, sp_dtype_t dt, int border, hipStream_t s) {
    return halo_launch(P, msg, g, c, dt, kPack, border, s);
}

int launch_halo_unpack(void *P, const void *msg, const Geo &g, int c, sp_dtype_t dt, int border, hipStream_t s) {
    return halo_launch(msg, P, g, c, dt, kUnpack, border, s);
}

int launch_halo_exchange(void *P, const Geo &g, int c, sp_dtype_t dt, int border, hipStream_t s) {
    return halo_launch(P, P, g, c, dt, kExchange, border, s);
}

// One-bit ReLU mask of a bf16 tensor.  Four lanes share a record of 32 channels (16 bytes each, so a wave reads
// a contiguous kilobyte); lane q holds channels 8 q .. 8 q + 7, of which the first four go to bits 4 q .. 4 q + 3
// of the record's low 16-bit word and the last four to the same bits of the high one (the order in which the
// matrix-core kernels produce and consume the bits).  The four contributions are OR-ed across the lanes.
__global__ __launch_bounds__(kThreads) void relu_bits_kernel(const u32x4 *__restrict__ y, uint32_t *__restrict__ bits,
                                                             size_t blocks) {
    const size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    const size_t rec = i >> 2;
    const int q = static_cast<int>(i & 3);
    uint32_t word = 0;
    if (rec < blocks) {
        const u32x4 v = y[i];
        uint32_t n = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            n |= positive<uint16_t>(static_cast<uint16_t>(v[k] & 0xffffu)) ? 1u << (2 * k) : 0u;
            n |= positive<uint16_t>(static_cast<uint16_t>(v[k] >> 16)) ? 2u << (2 * k) : 0u;
        }
        word = ((n & 0xfu) << (4 * q)) | ((n >> 4) << (16 + 4 * q));
    }
    word |= __shfl_xor(word, 1);
    word |= __shfl_xor(word, 2);
    if (q == 0 && rec < blocks) bits[rec] = word;
}

int launch_relu_bits(const void *y, void *bits, size_t blocks, hipStream_t s) {
    if (blocks == 0) return SP_OK;
    const size_t nblk = (blocks * 4 + kThreads - 1) / kThreads;
    if (nblk > 0x7fffffffULL) return SP_EGEOM;
    hipLaunchKernelGGL(relu_bits_kernel, dim3(static_cast<unsigned>(nblk)), dim3(kThreads), 0, s,
                       static_cast<const u32x4 *>(y), static_cast<uint32_t *>(bits), blocks);
    return record_hip(hipGetLastError());
}

int launch_relu_bwd(const void *dy, const void *y, void *dz, size_t elems, sp_dtype_t dt,
                    hipStream_t s) {
    if (elems == 0) return SP_OK;
    if (dt == SP_BF16 && elems % 8 == 0 && elems / 8 <= 0x7fffffffULL * kThreads) {
        const size_t nvec = elems / 8;
        hipLaunchKernelGGL(relu_bwd_bf16x8_kernel, dim3(static_cast<unsigned>((nvec + kThreads - 1) / kThreads)),
                           dim3(kThreads), 0, s, static_cast<const u32x4 *>(dy), static_cast<const u32x4 *>(y),
                           static_cast<u32x4 *>(dz), nvec);
        return record_hip(hipGetLastError());
    }
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
