// Instantiates the reduction kernels for element type bf16 (one translation
// unit per type so that they compile in parallel).
#include "mfr_kernels.hpp"

namespace mfr {

hipError_t launch_sum_bf16(const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream)
{
    return launch_sum<MFR_DTYPE_BF16>(p, grid, t, stream);
}

}  // namespace mfr
