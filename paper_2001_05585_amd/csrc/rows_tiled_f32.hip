// Tiled rows kernel, binary32 instances (one translation unit per element type: they compile in parallel).
#include "rows_tiled.hpp"

namespace mfr {

hipError_t launch_rows_tiled_f32(const void *x, unsigned long long rows, unsigned long long cols,
                                unsigned long long row_stride, float *out, const RowsTiledShape &s, unsigned grid,
                                bool nt, hipStream_t stream)
{
    return launch_rows_tiled_dt<MFR_DTYPE_F32>(x, rows, cols, row_stride, out, s, grid, nt, stream);
}

}  // namespace mfr
