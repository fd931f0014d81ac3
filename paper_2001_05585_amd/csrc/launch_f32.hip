// Instantiates the reduction kernels for element type f32 (one translation
// unit per type so that they compile in parallel).
#include "mfr_kernels.hpp"

namespace mfr {

hipError_t launch_sum_f32(const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream)
{
    return launch_sum<MFR_DTYPE_F32>(p, grid, t, stream);
}

}  // namespace mfr
