// The 3-D two-chunk convolution kernels (conv_mfma_pair_kernel.h) and the launch entry of both halves of the table.
#include "conv_mfma_pair_kernel.h"

namespace sp3d {

using namespace convk;

using PairKern = void (*)(ConvArgs);
// [mode][bias][epilogue] of the 2-D variant (conv_mfma_pair2d.hip)
const PairKern (&conv_mfma_pair_table_2d())[4][2][5];

namespace {

const PairKern (&table_3d())[4][2][5] {
    static const PairKern k[4][2][5] = SP3D_CONV_TABLE(wide::conv_mfma_pair_kernel, 3, kMaskBits, kReluBits);
    return k;
}

}  // namespace

hipError_t conv_mfma_pair_prepare() {
    for (int i = 0; i < 80; ++i) {
        const auto &k = i < 40 ? table_3d() : conv_mfma_pair_table_2d();
        // more than 64 KB of dynamic LDS has to be requested explicitly
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k[(i / 10) & 3][(i / 5) & 1][i % 5]),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, wide::LDS_BYTES);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

void conv_mfma_pair_launch(int flat, int mode, int bias, int epi, unsigned grid, hipStream_t s, const ConvArgs &a) {
    const auto &k = flat ? conv_mfma_pair_table_2d() : table_3d();
    hipLaunchKernelGGL(k[mode][bias][epi], dim3(grid), dim3(kThreads), wide::LDS_BYTES, s, a);
}

}  // namespace sp3d
