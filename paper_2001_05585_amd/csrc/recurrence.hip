// Variant #1 of the paper, "recurrence" (Section 5.1; Algorithms 1 and 2 with
// the chained MMAs of Section 4.3): every level turns each group of R * 512
// values into ONE value stored as binary16, and the host relaunches until one
// value is left.  Kept as the paper describes it, fp16 partials included, to
// show what the single-pass variant avoids: the partials overflow as soon as a
// group sum passes 65504 (Section 5.4).
//
// Per group (one wave each, the paper's geometry):
//   C_r = 1 x M_r + C_{r-1}, r = 1..R            fp32 accumulator, R MFMAs 16x16x32
//   A <- C_R                                      the 16 column sums, rounded to fp16
//   C_{R+1} = A x 1 + 0                           one MFMA 16x16x16: the group total in every entry
//   level_out[group] = (fp16) C_{R+1}[0][0]
#include "mfr_kernels.hpp"

namespace mfr {

typedef _Float16 half4 __attribute__((ext_vector_type(4)));

template <int R>
__global__ void __launch_bounds__(256) recurrence_level_kernel(const SumArgs a, unsigned short *level_out,
                                                               float *final_out)
{
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const unsigned wpb = blockDim.x >> 6;
    const unsigned long long c = (unsigned long long)blockIdx.x * wpb + wave;   // group index
    if (c >= a.chains) return;

    uint4v v[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const unsigned long long q = (c * R + r) * 64ull + lane;
        v[r] = load_slot_guarded<MFR_DTYPE_F16>(a, a.base, a.x, q, q < a.slots);
    }
    float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < R; ++r) acc = mma_ones<MFR_DTYPE_F16>(v[r], acc);

    // copy C to the A operand (Algorithm 2): lane l holds column sum (l mod 16);
    // A[i][k] = column sum k sits in lane l as k = 4 (l / 16) + 0..3
    const unsigned g = lane >> 4;
    half4 A;
#pragma unroll
    for (int k = 0; k < 4; ++k) A[k] = (_Float16)__shfl(acc.x, (int)(4u * g + (unsigned)k), 64);
    const _Float16 one = (_Float16)1.0f;
    const half4 ones = {one, one, one, one};
    const float4v zero = {0.f, 0.f, 0.f, 0.f};
    const float4v d = __builtin_amdgcn_mfma_f32_16x16x16f16(A, ones, zero, 0, 0, 0);
    if (lane == 0) {
        const _Float16 h = (_Float16)d.x;
        level_out[c] = __builtin_bit_cast(unsigned short, h);
        if (final_out) *final_out = (float)h;
    }
}

hipError_t launch_recurrence_level(const SumArgs &a, int R, unsigned short *level_out, float *final_out,
                                   hipStream_t stream)
{
    const unsigned wpb = 4;
    const unsigned long long blocks = (a.chains + wpb - 1) / wpb;
    if (blocks == 0 || blocks > 0x7fffffffull) return hipErrorInvalidValue;
    const dim3 g((unsigned)blocks), b(64 * wpb);
#define MFR_REC(R_) case R_: hipLaunchKernelGGL(recurrence_level_kernel<R_>, g, b, 0, stream, a, level_out, final_out); break;
    switch (R) {
        MFR_REC(1) MFR_REC(2) MFR_REC(3) MFR_REC(4) MFR_REC(5) MFR_REC(6) MFR_REC(7) MFR_REC(8)
    default: return hipErrorInvalidValue;
    }
#undef MFR_REC
    return hipGetLastError();
}

}  // namespace mfr
