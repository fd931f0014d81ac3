// Many short rows: sixteen row sums per MFMA chain.
//
// The ones-matrix product of Section 4.1 (eq. MMA1) yields one sum per column
// of the data operand.  For one long array all 16 columns belong to the same
// sum and are folded afterwards; here each column is given to a different row
// of a rows x cols array instead: lane l loads 8 consecutive values of row
// r0 + (l mod 16) at column c0 + 8 (l / 16), so that after the chain
// C_k = 1 x M_k + C_{k-1} (Section 4.3) along the columns, accumulator column
// j holds the complete sum of row r0 + j.  No fold, no cross-lane step: lane j
// of the first 16-lane row stores out[r0 + j].
//
// Requirements checked by the host: 16-bit element type, x 16-byte aligned,
// row stride a multiple of 8 elements.  cols is arbitrary (the last partial
// group of 8 values is read element-wise under a range check), rows too.
#include "mfr_kernels.hpp"

namespace mfr {

struct Rows16Args {
    const uint4v *base;              // first row, 16-byte aligned
    unsigned long long rows;
    unsigned long long cols;
    unsigned long long row_slots;    // row stride in 16-byte slots
    unsigned long long groups;       // ceil(rows / 16)
    float *out;
};

// Eight consecutive values of a row starting at column c (c is a multiple of 8).
template <bool NT>
__device__ __forceinline__ uint4v load_row_slot(const uint4v *row, unsigned long long c, unsigned long long cols,
                                                bool row_ok)
{
    uint4v r = {0u, 0u, 0u, 0u};
    if (!row_ok || c >= cols) return r;
    if (c + 8ull <= cols) return load_slot<NT>(row + c / 8ull);
    const unsigned short *e = (const unsigned short *)row;
    unsigned int h[8];
#pragma unroll
    for (unsigned k = 0; k < 8; ++k) {
        const bool ok = c + k < cols;
        const unsigned int t = e[ok ? c + k : c];      // c < cols: always readable
        h[k] = ok ? t : 0u;
    }
    r.x = h[0] | (h[1] << 16);
    r.y = h[2] | (h[3] << 16);
    r.z = h[4] | (h[5] << 16);
    r.w = h[6] | (h[7] << 16);
    return r;
}

// D: tiles (MFMAs) whose loads are issued together.
template <int DT, int D, bool NT>
__global__ void __launch_bounds__(1024) rows16_kernel(const Rows16Args a)
{
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const unsigned wpb = blockDim.x >> 6;
    const unsigned long long W = (unsigned long long)gridDim.x * wpb;
    const unsigned long long w = (unsigned long long)blockIdx.x * wpb + wave;
    const unsigned col_lane = 8u * (lane >> 4);          // this lane's column offset inside a 32-column tile
    const unsigned long long whole = a.cols / (32ull * D) * (32ull * D);   // columns covered by unmasked batches

    for (unsigned long long g = w; g < a.groups; g += W) {
        const unsigned long long r = g * 16ull + (lane & 15u);
        const bool row_ok = r < a.rows;
        const uint4v *row = a.base + (row_ok ? r : 0ull) * a.row_slots;
        float4v acc = {0.f, 0.f, 0.f, 0.f};                               // C_0 = 0
        unsigned long long c0 = 0;
        for (; c0 < whole; c0 += 32ull * D) {
            uint4v v[D];
#pragma unroll
            for (int d = 0; d < D; ++d)
                v[d] = row_ok ? load_slot<NT>(row + (c0 + 32ull * d + col_lane) / 8ull) : uint4v{0u, 0u, 0u, 0u};
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int d = 0; d < D; ++d) acc = mma_ones<DT>(v[d], acc);
        }
        if (c0 < a.cols) {                                                // ragged end of the rows
            uint4v v[D];
#pragma unroll
            for (int d = 0; d < D; ++d) v[d] = load_row_slot<NT>(row, c0 + 32ull * d + col_lane, a.cols, row_ok);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int d = 0; d < D; ++d) acc = mma_ones<DT>(v[d], acc);
        }
        if (lane < 16u && row_ok) a.out[r] = acc.x;
    }
}

// Rows of at most 32 * D columns: a group of 16 rows is one batch of D tiles, and GF
// groups are in flight together (GF * D loads per lane before the first MFMA).
template <int DT, int D, int GF, bool NT>
__global__ void __launch_bounds__(1024) rows16_short_kernel(const Rows16Args a)
{
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const unsigned wpb = blockDim.x >> 6;
    const unsigned long long W = (unsigned long long)gridDim.x * wpb;
    const unsigned long long w = (unsigned long long)blockIdx.x * wpb + wave;
    const unsigned col_lane = 8u * (lane >> 4);

    for (unsigned long long g0 = w; g0 < a.groups; g0 += (unsigned long long)GF * W) {
        uint4v v[GF][D];
        unsigned long long r[GF];
#pragma unroll
        for (int u = 0; u < GF; ++u) {
            const unsigned long long g = g0 + (unsigned long long)u * W;
            r[u] = g * 16ull + (lane & 15u);
            const bool row_ok = g < a.groups && r[u] < a.rows;
            const uint4v *row = a.base + (row_ok ? r[u] : 0ull) * a.row_slots;
#pragma unroll
            for (int d = 0; d < D; ++d) v[u][d] = load_row_slot<NT>(row, 32ull * d + col_lane, a.cols, row_ok);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < GF; ++u) {
            float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int d = 0; d < D; ++d) acc = mma_ones<DT>(v[u][d], acc);
            const unsigned long long g = g0 + (unsigned long long)u * W;
            if (lane < 16u && g < a.groups && r[u] < a.rows) a.out[r[u]] = acc.x;
        }
    }
}

template <int DT>
static hipError_t launch_rows16_t(const Rows16Args &a, unsigned grid, unsigned block, int tiles_in_flight,
                                  hipStream_t stream)
{
    const dim3 g(grid), b(block);
    if (a.cols <= 32) { hipLaunchKernelGGL((rows16_short_kernel<DT, 1, 8, true>), g, b, 0, stream, a); return hipGetLastError(); }
    if (a.cols <= 64) { hipLaunchKernelGGL((rows16_short_kernel<DT, 2, 4, true>), g, b, 0, stream, a); return hipGetLastError(); }
    if (a.cols <= 128) { hipLaunchKernelGGL((rows16_short_kernel<DT, 4, 2, true>), g, b, 0, stream, a); return hipGetLastError(); }
    switch (tiles_in_flight) {
    case 1: hipLaunchKernelGGL((rows16_kernel<DT, 1, true>), g, b, 0, stream, a); break;
    case 2: hipLaunchKernelGGL((rows16_kernel<DT, 2, true>), g, b, 0, stream, a); break;
    case 4: hipLaunchKernelGGL((rows16_kernel<DT, 4, true>), g, b, 0, stream, a); break;
    case 8: hipLaunchKernelGGL((rows16_kernel<DT, 8, true>), g, b, 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_rows16(int dtype, const void *x, unsigned long long rows, unsigned long long cols,
                         unsigned long long row_stride, float *out, unsigned grid, unsigned block,
                         int tiles_in_flight, hipStream_t stream)
{
    Rows16Args a;
    a.base = (const uint4v *)x;
    a.rows = rows;
    a.cols = cols;
    a.row_slots = row_stride / 8ull;
    a.groups = (rows + 15ull) / 16ull;
    a.out = out;
    if (dtype == MFR_DTYPE_F16) return launch_rows16_t<MFR_DTYPE_F16>(a, grid, block, tiles_in_flight, stream);
    if (dtype == MFR_DTYPE_BF16) return launch_rows16_t<MFR_DTYPE_BF16>(a, grid, block, tiles_in_flight, stream);
    return hipErrorInvalidValue;
}

}  // namespace mfr
