// Branch mode of the matrix-core convolution, pad mode 0 (a tap outside the image is -1 everywhere): its own
// translation unit so that the big kernel's instances compile in parallel.
#include "conv_mfma_fp4_kernel.h"

namespace bcnn {

hipError_t launch_branch_mfma_pad_minus(const MfmaArgs& a, const BranchArgs& b, const BranchEp& bp, int kind,
                                     hipStream_t stream)
{
    return launch_branch_mfma_kind<0>(a, b, bp, kind, stream);
}

}  // namespace bcnn
