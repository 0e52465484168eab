// Layers with few input channels on the matrix cores: the input tensor and the weights are copied with their
// input-channel axis zero-padded to a multiple of 32 (into the workspace), the matrix-core kernels run on the
// copies, and the weight gradient drops the padding rows again.  The zero channels contribute exact zeros, so
// the results are those of the unpadded contraction with the same fp32 accumulation.  The copies are plain
// HBM-bound sweeps (one 16-byte store per thread).
#include "common.h"

namespace sp3d {

namespace {

constexpr int kThreads = 256;

// out[v][c] = in[v][c] for c < cin, 0 for cin <= c < cp; one thread per (voxel, group of 8 output channels)
__global__ __launch_bounds__(kThreads) void pad_channels_kernel(const uint16_t *__restrict__ in, uint4 *__restrict__ out,
                                                                long long ngroups, int cin, int cp8) {
    const long long i = 1LL * blockIdx.x * kThreads + threadIdx.x;
    if (i >= ngroups) return;
    const long long v = i / cp8;
    const int c0 = static_cast<int>(i % cp8) * 8;
    const uint16_t *src = in + v * cin;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t lo = c0 + 2 * e < cin ? src[c0 + 2 * e] : 0u;
        const uint32_t hi = c0 + 2 * e + 1 < cin ? src[c0 + 2 * e + 1] : 0u;
        w[e] = lo | (hi << 16);
    }
    out[i] = make_uint4(w[0], w[1], w[2], w[3]);
}

// wp[t][ci][co] = w[t][ci][co] for ci < cin, 0 for the padding rows
__global__ __launch_bounds__(kThreads) void pad_weight_rows_kernel(const uint16_t *__restrict__ w, uint16_t *__restrict__ wp,
                                                                   int total, int cin, int cp, int cout) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int co = i % cout, ci = (i / cout) % cp, t = i / (cout * cp);
    wp[i] = ci < cin ? w[(static_cast<size_t>(t) * cin + ci) * cout + co] : static_cast<uint16_t>(0);
}

// dw[t][ci][co] = dwp[t][ci][co], ci < cin
__global__ __launch_bounds__(kThreads) void take_weight_rows_kernel(const float *__restrict__ dwp, float *__restrict__ dw,
                                                                    int total, int cin, int cp, int cout) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int co = i % cout, ci = (i / cout) % cin, t = i / (cout * cin);
    dw[i] = dwp[(static_cast<size_t>(t) * cp + ci) * cout + co];
}

}  // namespace

int padded_channels(int cin) { return (cin + 31) / 32 * 32; }

bool chan_pad_supported(const Geo &g, int cin, int cout, sp_dtype_t dt) {
    return dt == SP_BF16 && cin % 32 != 0 && cin <= 1024 && cout % 32 == 0 &&
           conv_mfma_supported(g, padded_channels(cin), cout, dt) &&
           wgrad_mfma_supported(g, padded_channels(cin), cout, dt);
}

// workspace layout: [padded tensor][padded weights (forward) or padded weight gradient (wgrad)][the kernels' own]
static size_t tensor_bytes(const Geo &g, int cp) {
    return (static_cast<size_t>(g.ntiles) * g.tile_vox * cp * 2 + 255) / 256 * 256;
}
static size_t weight_bytes(const Geo &g, int cp, int cout, size_t es) {
    return (static_cast<size_t>(taps_of(g)) * cp * cout * es + 255) / 256 * 256;
}

size_t chan_pad_fwd_ws_bytes(const Geo &g, int cin, int cout) {
    const int cp = padded_channels(cin);
    return tensor_bytes(g, cp) + weight_bytes(g, cp, cout, 2) + conv_mfma_ws_bytes(g, cp, cout);
}

size_t chan_pad_wgrad_ws_bytes(const Geo &g, int cin, int cout) {
    const int cp = padded_channels(cin);
    return tensor_bytes(g, cp) + weight_bytes(g, cp, cout, 4) + wgrad_mfma_ws_bytes(g, cp, cout);
}

static int pad_tensor(const void *Px, void *dst, const Geo &g, int cin, int cp, hipStream_t s) {
    const long long ngroups = 1LL * g.ntiles * g.tile_vox * (cp / 8);
    const long long blocks = (ngroups + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return SP_EGEOM;
    hipLaunchKernelGGL(pad_channels_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, s,
                       static_cast<const uint16_t *>(Px), static_cast<uint4 *>(dst), ngroups, cin, cp / 8);
    return record_hip(hipGetLastError());
}

int launch_conv_chan_pad_fwd(const void *Px, const void *w, const float *bias, void *Py, const Geo &g, int cin,
                             int cout, bool relu, void *ws, hipStream_t s) {
    const int cp = padded_channels(cin);
    char *base = static_cast<char *>(ws);
    void *xp = base, *wp = base + tensor_bytes(g, cp), *inner = base + tensor_bytes(g, cp) + weight_bytes(g, cp, cout, 2);
    int rc = pad_tensor(Px, xp, g, cin, cp, s);
    if (rc != SP_OK) return rc;
    const int total = taps_of(g) * cp * cout;
    hipLaunchKernelGGL(pad_weight_rows_kernel, dim3((total + kThreads - 1) / kThreads), dim3(kThreads), 0, s,
                       static_cast<const uint16_t *>(w), static_cast<uint16_t *>(wp), total, cin, cp, cout);
    rc = record_hip(hipGetLastError());
    if (rc != SP_OK) return rc;
    return launch_conv_mfma(xp, wp, bias, Py, g, cp, cout, relu, false, inner, s);
}

int launch_wgrad_chan_pad(const void *Px, const void *Pdz, float *dw, float *db, const Geo &g, int cin, int cout,
                          sp_dtype_t dt, void *ws, hipStream_t s) {
    const int cp = padded_channels(cin);
    char *base = static_cast<char *>(ws);
    void *xp = base;
    float *dwp = reinterpret_cast<float *>(base + tensor_bytes(g, cp));
    void *inner = base + tensor_bytes(g, cp) + weight_bytes(g, cp, cout, 4);
    int rc = pad_tensor(Px, xp, g, cin, cp, s);
    if (rc != SP_OK) return rc;
    rc = launch_wgrad_mfma(shifted(static_cast<const void *>(xp), g, cp, dt), shifted(Pdz, g, cout, dt), dwp, db, g, cp,
                           cout, inner, s);
    if (rc != SP_OK) return rc;
    const int total = taps_of(g) * cin * cout;
    hipLaunchKernelGGL(take_weight_rows_kernel, dim3((total + kThreads - 1) / kThreads), dim3(kThreads), 0, s, dwp, dw,
                       total, cin, cp, cout);
    return record_hip(hipGetLastError());
}

}  // namespace sp3d
