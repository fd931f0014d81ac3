// Context only, never on the library's path: the vendor's device-wide reduction (hipCUB) on the same
// fp16 inputs, as the counterpart of the CUB comparison in Section 6 of the paper.  Built into a separate
// shared library (libmfrcontext.so) that only the benchmark sweeps load.
//   ctx_hipcub_sum_f16_f32acc  fp16 values converted to float on load, float accumulation ("CUB-float")
//   ctx_hipcub_sum_f16         fp16 accumulation ("CUB-half"; overflows past 65504, as the paper notes)
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <hipcub/hipcub.hpp>

namespace {
struct HalfToFloat {
    __host__ __device__ float operator()(const __half &h) const { return __half2float(h); }
};
}  // namespace

extern "C" {

// temp == nullptr: writes the scratch size needed to *temp_bytes and returns.
int ctx_hipcub_sum_f16_f32acc(const void *x, size_t n, float *out, void *temp, size_t *temp_bytes, hipStream_t stream)
{
    hipcub::TransformInputIterator<float, HalfToFloat, const __half *> it((const __half *)x, HalfToFloat());
    return (int)hipcub::DeviceReduce::Sum(temp, *temp_bytes, it, out, (int)n, stream);
}

int ctx_hipcub_sum_f16(const void *x, size_t n, void *out_half, void *temp, size_t *temp_bytes, hipStream_t stream)
{
    return (int)hipcub::DeviceReduce::Sum(temp, *temp_bytes, (const __half *)x, (__half *)out_half, (int)n, stream);
}

}  // extern "C"
