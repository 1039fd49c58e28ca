// Branch mode of the matrix-core convolution, pad mode 1 (the branch's pad words): its own
// translation unit so that the big kernel's instances compile in parallel.
#include "conv_mfma_fp4_kernel.h"

namespace bcnn {

hipError_t launch_branch_mfma_pad_words(const MfmaArgs& a, const BranchArgs& b, const BranchEp& bp, int kind,
                                     hipStream_t stream)
{
    return launch_branch_mfma_kind<1>(a, b, bp, kind, stream);
}

}  // namespace bcnn
