// The two-chunk convolution kernels of the 2-D variant (kernel extent 1 along D; conv_mfma_pair_kernel.h).
#include "conv_mfma_pair_kernel.h"

namespace sp3d {

using namespace convk;

using PairKern = void (*)(ConvArgs);

// [mode][bias][epilogue]; the 2-D variant has no bit forms of the epilogue (the host refuses them)
const PairKern (&conv_mfma_pair_table_2d())[4][2][5] {
    static const PairKern k[4][2][5] = SP3D_CONV_TABLE(wide::conv_mfma_pair_kernel, 1, kNone, kNone);
    return k;
}

}  // namespace sp3d
