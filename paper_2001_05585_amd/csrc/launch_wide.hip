// Higher-accuracy mode of the single-pass reduction: the chains of R MFMAs keep
// their fp32 accumulators (Section 4.3), but everything after a chain is done
// in binary64 -- each lane adds its chain's column sum to a binary64 running
// sum, lanes, waves and blocks are combined in binary64, and the result is
// returned as a double.  The only fp32 roundings left are the 32 R additions
// inside each accumulator column, so the error no longer grows with n.  (The
// paper discusses the precision of the fp32 partials in Sections 2.2 and 5.4;
// this mode removes the part of the error that comes from combining them.)
#include "mfr_kernels.hpp"

namespace mfr {

// All threads of one block: sum of partials[0..count) in fixed order; thread 0 gets it.
__device__ __forceinline__ double block_sum_of_doubles(const double *partials, unsigned int count, double *lds)
{
    const unsigned int lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, wpb = (blockDim.x + 63u) >> 6;
    double t = 0.0;
    for (unsigned int i = threadIdx.x; i < count; i += blockDim.x)
        t += __hip_atomic_load(&partials[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    t = wave64_sum_f64(t);
    if (lane == 0) lds[wave] = t;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0)
        for (unsigned int w = 0; w < wpb; ++w) total += lds[w];
    return total;
}

template <int R, int U, bool NT>
__global__ void __launch_bounds__(1024) sum_kernel_wide(const SumArgs a)
{
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const unsigned wpb = (blockDim.x + 63u) >> 6;
    const unsigned long long W = (unsigned long long)gridDim.x * wpb;
    const unsigned long long w = (unsigned long long)blockIdx.x * wpb + wave;

    // lane l: binary64 running sum of column (l mod 16) over all of this wave's chains
    const double column = stream_chains<KIND_MFMA_COLUMNS, MFR_DTYPE_F16, R, U, NT, false, double>(
        a, a.base, a.x, lane, w, a.chains, W, w == W - 1);
    const double wave_total = row16_sum_f64(column);     // the four 16-lane rows hold copies

    __shared__ double wave_partials[kMaxWavesPerBlock];
    __shared__ double combine_lds[kMaxWavesPerBlock];
    if (lane == 0) wave_partials[wave] = wave_total;
    __syncthreads();
    double block_sum = 0.0;
    if (threadIdx.x == 0)
        for (unsigned int i = 0; i < wpb; ++i) block_sum += wave_partials[i];

    double *out = (double *)a.out;
    if (gridDim.x == 1) {
        if (threadIdx.x == 0) *out = block_sum;
        return;
    }
    if (a.combine_slots == nullptr) {
        if (threadIdx.x == 0) ((double *)a.partials)[blockIdx.x] = block_sum;
        return;
    }
    // the same hand-over as in the fp32 kernel, with 64-bit slots
    unsigned long long *slots = (unsigned long long *)a.combine_slots;
    if (blockIdx.x + 1u != gridDim.x) {
        if (threadIdx.x == 0) publish_slot(&slots[blockIdx.x], block_sum);
        return;
    }
    const double others = gather_slots(slots, gridDim.x - 1u, combine_lds);
    if (threadIdx.x == 0) *out = others + block_sum;
}

__global__ void __launch_bounds__(256) combine_wide_kernel(const double *partials, unsigned int count, double *out)
{
    __shared__ double lds[kMaxWavesPerBlock];
    const double total = block_sum_of_doubles(partials, count, lds);
    if (threadIdx.x == 0) *out = total;
}

template <int R, int U>
static hipError_t launch_wide_ru(const Plan &p, dim3 grid, bool nt, hipStream_t stream)
{
    const dim3 b((unsigned)p.threads);
    if (nt) hipLaunchKernelGGL((sum_kernel_wide<R, U, true>), grid, b, 0, stream, p.a);
    else hipLaunchKernelGGL((sum_kernel_wide<R, U, false>), grid, b, 0, stream, p.a);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && grid.x > 1 && p.a.combine_slots == nullptr) {
        hipLaunchKernelGGL(combine_wide_kernel, dim3(1), dim3(256), 0, stream, (const double *)p.a.partials, grid.x,
                           (double *)p.a.out);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_sum_wide(const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream)
{
    if (p.half) return hipErrorInvalidValue;
    const bool nt = t.nontemporal == 2;
#define MFR_CASE(R_, U_) case (R_) * 16 + (U_): return launch_wide_ru<R_, U_>(p, grid, nt, stream);
    switch (t.chain_R * 16 + t.chains_in_flight) {
        MFR_CASE(1, 1) MFR_CASE(1, 2) MFR_CASE(1, 3) MFR_CASE(1, 4) MFR_CASE(1, 6) MFR_CASE(1, 8)
        MFR_CASE(2, 1) MFR_CASE(2, 2) MFR_CASE(2, 3) MFR_CASE(2, 4) MFR_CASE(2, 6) MFR_CASE(2, 8)
        MFR_CASE(3, 1) MFR_CASE(3, 2) MFR_CASE(3, 3) MFR_CASE(3, 4)
        MFR_CASE(4, 1) MFR_CASE(4, 2) MFR_CASE(4, 3) MFR_CASE(4, 4)
        MFR_CASE(5, 1) MFR_CASE(5, 2) MFR_CASE(5, 3)
        MFR_CASE(6, 1) MFR_CASE(6, 2)
        MFR_CASE(7, 1) MFR_CASE(7, 2)
        MFR_CASE(8, 1) MFR_CASE(8, 2)
    default: return hipErrorInvalidValue;
    }
#undef MFR_CASE
}

}  // namespace mfr
