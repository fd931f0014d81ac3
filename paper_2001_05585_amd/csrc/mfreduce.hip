// libmfreduce: sum of n fp16 values to one fp32 on gfx950 (MI355X).
//
// Single-pass reduction (paper Section 5.2) in three levels:
//   1. every wavefront runs chains of R MFMAs  C_r = 1 x M_r + C_{r-1}
//      (Section 4.3) on 16x16x32 fp16 tiles with an fp32 accumulator, and
//      folds each finished chain to one fp32 partial;
//   2. the waves of a block combine their partials through LDS;
//   3. block partials go to a scratch array; the block that draws the last
//      ticket adds them in index order and writes the result (the paper adds
//      them with float atomics, whose order varies from run to run).
// A conventional kernel (per-lane fp32 accumulation + wave shuffle tree, the
// comparison kernel of Section 5.4) shares levels 2 and 3.
//
// Memory view.  The input is addressed in 16-byte "slots" counted from x
// rounded down to a 16-byte boundary.  Slot 0 may start before x (head
// padding) and the last slot may end after x + n; those two are read
// element-wise under a range check, padding contributes +0 (the border
// handling Section 4.1 leaves to the implementation).  All other slots are
// read with one 128-bit load per lane, 64 lanes = 1 KiB contiguous per load
// instruction = one MFMA B operand (8 halves per lane).  Any assignment of
// elements to operand positions yields the same total, so the layout is chosen
// for coalescing alone.

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <utility>

#include "mfreduce.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

constexpr int kMaxWavesPerBlock = 16;

struct SumArgs {
    const uint4v *base;          // x rounded down to 16 bytes: slot 0
    const unsigned short *x;     // first element
    unsigned long long n;        // element count
    unsigned long long vend;     // head + n: end of the valid range in slot-relative elements
    unsigned long long main0;    // first slot of the unmasked main region
    unsigned long long chains;   // number of full chains in the main region
    unsigned long long epi0;     // epilogue positions [epi0, epi1)
    unsigned long long epi1;
    unsigned long long slots;    // total slots covering [x, x + n)
    unsigned int head;           // elements of slot 0 that lie before x (0..7)
    float *partials;             // one per block
    unsigned int *ticket;
    float *out;
};

// ---------------------------------------------------------------- loads ---

template <bool NT>
__device__ __forceinline__ uint4v load_slot(const uint4v *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

// Slot q with every element range-checked against [x, x + n).  A slot that
// lies wholly inside is one 128-bit load; a straddling slot is read with eight
// independent 16-bit loads whose indices are clamped into range, so that all
// of them are in flight together, and out-of-range elements are replaced by +0.
__device__ __forceinline__ uint4v load_slot_guarded(const SumArgs &a, unsigned long long q, bool active)
{
    const unsigned long long v0 = q * 8ull;
    const bool full = active && v0 >= a.head && v0 + 8ull <= a.vend;
    uint4v r = {0u, 0u, 0u, 0u};
    if (full) r = a.base[q];
    if (active && !full) {
        unsigned int h[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const unsigned long long v = v0 + (unsigned)k;
            const bool ok = v >= a.head && v < a.vend;
            const unsigned int t = a.x[ok ? v - a.head : 0ull];   // n >= 1: x[0] is readable
            h[k] = ok ? t : 0u;
        }
        r.x = h[0] | (h[1] << 16);
        r.y = h[2] | (h[3] << 16);
        r.z = h[4] | (h[5] << 16);
        r.w = h[6] | (h[7] << 16);
    }
    return r;
}

// Epilogue position p -> slot: positions past the last slot stand for slot 0
// (the head slot is skipped by the main region and picked up here); positions
// at or past epi1 yield zeros.
__device__ __forceinline__ uint4v load_epilogue(const SumArgs &a, unsigned long long p, bool carries)
{
    return load_slot_guarded(a, p < a.slots ? p : 0ull, carries && p < a.epi1);
}

// ------------------------------------------------------- lane exchanges ---

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
    return v + __int_as_float(t);
}

// Sum over each row of 16 lanes, result in every lane of the row.
__device__ __forceinline__ float row16_sum(float v)
{
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror
    v = dpp_add<0x140>(v);   // row_mirror
    return v;
}

// Sum over the 64 lanes, wave-uniform.
__device__ __forceinline__ float wave64_sum(float v)
{
    v = row16_sum(v);
    const float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (a + b) + (c + d);
}

__device__ __forceinline__ double wave64_sum_f64(double v)
{
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// All threads of one block: sum of partials[0..count) in binary64, fixed order
// (thread t takes t, t + blockDim, ... with four running sums, then lanes, then
// waves).  Loads are device-scope atomic loads so that values published by
// other compute dies are observed.  Result valid in thread 0.
__device__ __forceinline__ double block_sum_f64(const float *partials, unsigned int count, double *lds)
{
    const unsigned int lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, wpb = (blockDim.x + 63u) >> 6;
    double t0 = 0.0, t1 = 0.0, t2 = 0.0, t3 = 0.0;
    const unsigned int step = blockDim.x;
    unsigned int i = threadIdx.x;
    for (; i + 3u * step < count; i += 4u * step) {
        const float p0 = __hip_atomic_load(&partials[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float p1 = __hip_atomic_load(&partials[i + step], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float p2 = __hip_atomic_load(&partials[i + 2u * step], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float p3 = __hip_atomic_load(&partials[i + 3u * step], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        t0 += (double)p0; t1 += (double)p1; t2 += (double)p2; t3 += (double)p3;
    }
    for (; i < count; i += step)
        t0 += (double)__hip_atomic_load(&partials[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    double t = wave64_sum_f64((t0 + t1) + (t2 + t3));
    if (lane == 0) lds[wave] = t;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0)
        for (unsigned int w = 0; w < wpb; ++w) total += lds[w];
    return total;
}

// ------------------------------------------------------ tile consumers ---

// One MFMA of the chain: C = 1 x M + C  (Section 4.3).  A is the all-ones
// 16x32 operand, B the 32x16 data tile; every row of C then holds the 16
// column sums, i.e. lane l holds column (l mod 16) in each of its 4 registers.
__device__ __forceinline__ float4v mma_ones(uint4v tile, float4v c)
{
    const _Float16 one = (_Float16)1.0f;
    const half8 ones = {one, one, one, one, one, one, one, one};
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, __builtin_bit_cast(half8, tile), c, 0, 0, 0);
}

// Chain total from the accumulator: the 16 distinct column sums sit in one
// register across the 16 lanes of a row (all rows and registers are copies),
// so an fp32 row fold replaces the final "x ones" MMA and keeps the chain
// result in fp32 (the accumulator is never rounded to fp16).
__device__ __forceinline__ float chain_total(float4v c)
{
    return row16_sum(c.x);
}

// Conventional path: fp32 sum of the 8 halves of one slot.
__device__ __forceinline__ float slot_sum_f32(uint4v s)
{
    const half8 h = __builtin_bit_cast(half8, s);
    return (((float)h[0] + (float)h[1]) + ((float)h[2] + (float)h[3])) +
           (((float)h[4] + (float)h[5]) + ((float)h[6] + (float)h[7]));
}

// One chain of R tiles to one fp32 value.  MFMA path: the chain total, uniform
// over the wave.  Conventional path: this lane's share of it.
template <int KERNEL, int R>
__device__ __forceinline__ float consume_chain(const uint4v (&v)[R])
{
    if constexpr (KERNEL == MFR_KERNEL_MFMA) {
        float4v acc = {0.f, 0.f, 0.f, 0.f};                 // C_0 = 0
#pragma unroll
        for (int r = 0; r < R; ++r) acc = mma_ones(v[r], acc);
        return chain_total(acc);
    } else {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r) s += slot_sum_f32(v[r]);
        return s;
    }
}

// ------------------------------------------------------------- kernels ---

// KERNEL: MFR_KERNEL_MFMA or MFR_KERNEL_SHFL.  R: chain length.  U: chains in
// flight.  NT: non-temporal loads.  HALF: only lanes 0..31 carry data (the
// "32-thread block" geometry on a wave64 machine), a tile is then 32 slots.
template <int KERNEL, int R, int U, bool NT, bool HALF>
__global__ void __launch_bounds__(1024) sum_kernel(const SumArgs a)
{
    constexpr unsigned TS = HALF ? 32u : 64u;          // slots per tile
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform
    const unsigned wpb = (blockDim.x + 63u) >> 6;
    const unsigned long long W = (unsigned long long)gridDim.x * wpb;
    const unsigned long long w = (unsigned long long)blockIdx.x * wpb + wave;
    const bool carries = !HALF || lane < 32u;
    const uint4v zero4 = {0u, 0u, 0u, 0u};

    // MFMA path: `partial` is the wave's running sum of chain totals (uniform).
    // SHFL path: `partial` is this lane's running fp32 sum.
    float partial = 0.f;
    const uint4v *lane_base = a.base + a.main0 + (carries ? lane : 0u);

    unsigned long long c = w;
    if constexpr (U > 1) {
        for (; c + (unsigned long long)(U - 1) * W < a.chains; c += (unsigned long long)U * W) {
            uint4v v[U][R];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const uint4v *p = lane_base + ((c + (unsigned long long)u * W) * R + r) * TS;
                    v[u][r] = carries ? load_slot<NT>(p) : zero4;
                }
            // all U * R loads are issued before the first is consumed
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < U; ++u) partial += consume_chain<KERNEL, R>(v[u]);
        }
    }
    for (; c < a.chains; c += W) {
        uint4v v[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint4v *p = lane_base + (c * R + r) * TS;
            v[r] = carries ? load_slot<NT>(p) : zero4;
        }
        __builtin_amdgcn_sched_barrier(0);
        partial += consume_chain<KERNEL, R>(v);
    }

    // Border: leftover whole tiles (fewer than R), leftover slots, the partial
    // last slot and the head slot, as masked tiles in chains of R (at most two
    // chains; tiles past the end are all zeros).
    if (w == W - 1) {
        for (unsigned long long p0 = a.epi0; p0 < a.epi1; p0 += (unsigned long long)R * TS) {
            uint4v v[R];
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = load_epilogue(a, p0 + (unsigned long long)r * TS + lane, carries);
            partial += consume_chain<KERNEL, R>(v);
        }
    }

    if constexpr (KERNEL == MFR_KERNEL_SHFL) partial = wave64_sum(partial);

    // Level 2: one value per block from its wave partials.
    __shared__ float wave_partials[kMaxWavesPerBlock];
    __shared__ double wave_partials_f64[kMaxWavesPerBlock];
    __shared__ unsigned int is_last;
    if (lane == 0) wave_partials[wave] = partial;
    __syncthreads();
    float block_sum = 0.f;
    if (wave == 0) {
        const float t = lane < wpb ? wave_partials[lane] : 0.f;
        block_sum = row16_sum(t);      // wpb <= 16: all partials sit in row 0
    }

    // Level 3: all block partials to one value, in index order.
    if (gridDim.x == 1) {
        if (threadIdx.x == 0) *a.out = block_sum;
        return;
    }
    if (a.ticket == nullptr) {
        // two-launch combine: the partial is picked up by combine_kernel
        if (threadIdx.x == 0) a.partials[blockIdx.x] = block_sum;
        return;
    }
    // Single-launch combine.  A release fence at device scope costs a write-back
    // of the whole L2 per block, so ordering is obtained from the atomics
    // themselves: the partial is published with a returning device-scope
    // exchange, and the ticket is drawn only after that exchange has returned,
    // i.e. after it has been performed at the device's coherence point.  The
    // block that draws the last ticket therefore finds every partial there.
    if (threadIdx.x == 0) {
        unsigned int prev = __hip_atomic_exchange((unsigned int *)&a.partials[blockIdx.x],
                                                  __float_as_uint(block_sum), __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
        // the exchange result must be in a register (waits for it) and no later
        // memory operation may be moved above this point
        asm volatile("" : "+v"(prev) : : "memory");
        // wraps to 0 after the last block, so the counter is ready for the next call
        const unsigned int old = atomicInc(a.ticket, gridDim.x - 1u);
        is_last = (old == gridDim.x - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;
    const double total = block_sum_f64(a.partials, gridDim.x, wave_partials_f64);
    if (threadIdx.x == 0) *a.out = (float)total;
}

// Second launch of the two-launch combine: one block adds all block partials.
__global__ void __launch_bounds__(1024) combine_kernel(const float *partials, unsigned int count, float *out)
{
    __shared__ double wave_partials_f64[kMaxWavesPerBlock];
    const double total = block_sum_f64(partials, count, wave_partials_f64);
    if (threadIdx.x == 0) *out = (float)total;
}

__global__ void store_zero_kernel(float *out) { *out = 0.f; }

// ------------------------------------------------------------ host side ---

thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e, const char *what)
{
    snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", what, hipGetErrorString(e));
    return MFR_ERR_HIP;
}

#define MFR_HIP(call)                                   \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) return hip_fail(e_, #call); \
    } while (0)

struct DeviceInfo {
    bool known = false;
    bool gfx950 = false;
    int cus = 0;
};

struct Scratch {
    float *partials = nullptr;
    unsigned int *ticket = nullptr;
    size_t capacity = 0;     // block partials
};

std::mutex g_mutex;
DeviceInfo g_devices[64];
std::map<std::pair<int, hipStream_t>, Scratch> g_scratch;

constexpr int kDefaultBlock = 256;
constexpr int kDefaultR = 4;
constexpr int kDefaultWavesPerCU = 4;
constexpr long long kTicketMaxBlocks = 320;    // larger grids combine with a second launch

int default_in_flight(int R)
{
    int u = 8 / R;
    if (u >= 8) return 8;
    if (u >= 4) return 4;
    if (u >= 2) return 2;
    return 1;
}

bool valid_block(int b)
{
    return b == 32 || b == 64 || b == 128 || b == 256 || b == 512 || b == 1024;
}

// Fills in defaults and checks ranges; no HIP calls.
int resolve_tuning(const mfr_tuning *in, mfr_tuning *t)
{
    mfr_tuning z;
    memset(&z, 0, sizeof z);
    if (in) z = *in;
    if (z.block_threads == 0) z.block_threads = kDefaultBlock;
    if (z.chain_R == 0) z.chain_R = kDefaultR;
    if (!valid_block(z.block_threads)) return MFR_ERR_INVALID_ARG;
    if (z.chain_R < 1 || z.chain_R > 8) return MFR_ERR_INVALID_ARG;
    if (z.grid_blocks < MFR_GRID_ONE_CHAIN) return MFR_ERR_INVALID_ARG;
    if (z.kernel != MFR_KERNEL_MFMA && z.kernel != MFR_KERNEL_SHFL) return MFR_ERR_INVALID_ARG;
    if (z.chains_in_flight == 0) z.chains_in_flight = default_in_flight(z.chain_R);
    const int u = z.chains_in_flight;
    if (!(u == 1 || u == 2 || u == 4 || u == 8)) return MFR_ERR_INVALID_ARG;
    if (u * z.chain_R > 16) return MFR_ERR_INVALID_ARG;
    if (z.nontemporal == 0) z.nontemporal = 2;
    if (z.nontemporal != 1 && z.nontemporal != 2) return MFR_ERR_INVALID_ARG;
    if (z.combine < 0 || z.combine > 2) return MFR_ERR_INVALID_ARG;
    *t = z;
    return MFR_OK;
}

struct Plan {
    SumArgs a;
    int threads;             // launched threads per block (>= 64)
    int waves;               // waves per block
    bool half;               // 32-thread geometry
    unsigned long long chains;
};

// Slot / chain arithmetic for n elements starting at byte address x_addr.
void plan_region(size_t n, size_t x_addr, const mfr_tuning &t, Plan *p)
{
    memset(p, 0, sizeof *p);
    p->half = t.block_threads == 32;
    p->threads = p->half ? 64 : t.block_threads;
    p->waves = p->threads / 64;
    const unsigned long long ts = p->half ? 32ull : 64ull;
    const unsigned int head = (unsigned int)((x_addr & 15u) / 2u);
    const unsigned long long vend = (unsigned long long)head + n;
    const unsigned long long slots = (vend + 7ull) / 8ull;
    const unsigned long long s0 = head ? 1ull : 0ull;
    const unsigned long long s1 = vend / 8ull;                 // slots that end at or before vend
    const unsigned long long full = s1 > s0 ? s1 - s0 : 0ull;
    const unsigned long long chains = full / (ts * (unsigned)t.chain_R);
    p->a.head = head;
    p->a.n = n;
    p->a.vend = vend;
    p->a.main0 = s0;
    p->a.chains = chains;
    p->a.epi0 = s0 + chains * ts * (unsigned)t.chain_R;
    p->a.epi1 = slots + (head ? 1ull : 0ull);
    if (p->a.epi0 > p->a.epi1) p->a.epi0 = p->a.epi1;          // n smaller than the head slot
    p->a.slots = slots;
    p->chains = chains;
}

int device_info(int dev, DeviceInfo *out)
{
    if (dev < 0 || dev >= 64) return MFR_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceInfo &d = g_devices[dev];
    if (!d.known) {
        hipDeviceProp_t prop;
        MFR_HIP(hipGetDeviceProperties(&prop, dev));
        d.gfx950 = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
        d.cus = prop.multiProcessorCount;
        d.known = true;
    }
    *out = d;
    return MFR_OK;
}

long long grid_blocks_for(const Plan &p, const mfr_tuning &t, int cus)
{
    const unsigned long long need = (p.chains + (unsigned)p.waves - 1ull) / (unsigned)p.waves;
    unsigned long long g;
    if (t.grid_blocks == MFR_GRID_ONE_CHAIN) {
        g = need;
    } else if (t.grid_blocks == MFR_GRID_AUTO) {
        int per_cu = kDefaultWavesPerCU / p.waves;
        if (per_cu < 1) per_cu = 1;
        g = (unsigned long long)cus * (unsigned)per_cu;
        if (g > need) g = need;
    } else {
        g = (unsigned long long)t.grid_blocks;
    }
    if (g < 1ull) g = 1ull;
    if (g > 0x7fffffffull) return -1;
    return (long long)g;
}

int get_scratch(int dev, hipStream_t stream, size_t blocks, Scratch *out)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    Scratch &s = g_scratch[std::make_pair(dev, stream)];
    if (s.capacity < blocks) {
        size_t cap = s.capacity ? s.capacity : 4096;
        while (cap < blocks) cap *= 2;
        if (s.partials) {
            // earlier calls on this stream may still be using the old buffers
            MFR_HIP(hipStreamSynchronize(stream));
            MFR_HIP(hipFree(s.partials));
            s.partials = nullptr;
            s.ticket = nullptr;
            s.capacity = 0;
        }
        void *mem = nullptr;
        MFR_HIP(hipMalloc(&mem, 256 + cap * sizeof(float)));
        // ticket at offset 0, partials at offset 256
        hipError_t e = hipMemset(mem, 0, 256);
        if (e != hipSuccess) { (void)hipFree(mem); return hip_fail(e, "hipMemset(scratch)"); }
        s.ticket = (unsigned int *)mem;
        s.partials = (float *)((char *)mem + 256);
        s.capacity = cap;
    }
    *out = s;
    return MFR_OK;
}

template <int KERNEL, int R, int U>
hipError_t launch_ru(const Plan &p, int grid, bool nt, hipStream_t stream)
{
    const dim3 g((unsigned)grid), b((unsigned)p.threads);
    if (p.half) {
        if (nt) hipLaunchKernelGGL((sum_kernel<KERNEL, R, U, true, true>), g, b, 0, stream, p.a);
        else hipLaunchKernelGGL((sum_kernel<KERNEL, R, U, false, true>), g, b, 0, stream, p.a);
    } else {
        if (nt) hipLaunchKernelGGL((sum_kernel<KERNEL, R, U, true, false>), g, b, 0, stream, p.a);
        else hipLaunchKernelGGL((sum_kernel<KERNEL, R, U, false, false>), g, b, 0, stream, p.a);
    }
    return hipGetLastError();
}

template <int KERNEL>
hipError_t launch_k(const Plan &p, int grid, const mfr_tuning &t, hipStream_t stream)
{
    const bool nt = t.nontemporal == 2;
#define MFR_CASE(R_, U_) \
    case (R_) * 16 + (U_): return launch_ru<KERNEL, R_, U_>(p, grid, nt, stream);
    switch (t.chain_R * 16 + t.chains_in_flight) {
        MFR_CASE(1, 1) MFR_CASE(1, 2) MFR_CASE(1, 4) MFR_CASE(1, 8)
        MFR_CASE(2, 1) MFR_CASE(2, 2) MFR_CASE(2, 4) MFR_CASE(2, 8)
        MFR_CASE(3, 1) MFR_CASE(3, 2) MFR_CASE(3, 4)
        MFR_CASE(4, 1) MFR_CASE(4, 2) MFR_CASE(4, 4)
        MFR_CASE(5, 1) MFR_CASE(5, 2)
        MFR_CASE(6, 1) MFR_CASE(6, 2)
        MFR_CASE(7, 1) MFR_CASE(7, 2)
        MFR_CASE(8, 1) MFR_CASE(8, 2)
    default: return hipErrorInvalidValue;
    }
#undef MFR_CASE
}

int sum_impl(const mfr_half *x, size_t n, float *out, const mfr_tuning *tin, hipStream_t stream)
{
    mfr_tuning t;
    const int st = resolve_tuning(tin, &t);
    if (st != MFR_OK) return st;
    if (!out) return MFR_ERR_INVALID_ARG;
    if (n > 0 && !x) return MFR_ERR_INVALID_ARG;
    if (((size_t)x & 1u) != 0) return MFR_ERR_INVALID_ARG;
    if (n > ((size_t)1 << 60)) return MFR_ERR_INVALID_ARG;

    int dev = 0;
    MFR_HIP(hipGetDevice(&dev));
    DeviceInfo info;
    const int ds = device_info(dev, &info);
    if (ds != MFR_OK) return ds;
    if (!info.gfx950) return MFR_ERR_UNSUPPORTED;

    if (n == 0) {
        hipLaunchKernelGGL(store_zero_kernel, dim3(1), dim3(1), 0, stream, out);
        MFR_HIP(hipGetLastError());
        return MFR_OK;
    }

    Plan p;
    plan_region(n, (size_t)x, t, &p);
    const long long grid = grid_blocks_for(p, t, info.cus);
    if (grid < 1) return MFR_ERR_INVALID_ARG;

    Scratch s;
    if (grid > 1) {
        const int ss = get_scratch(dev, stream, (size_t)grid, &s);
        if (ss != MFR_OK) return ss;
    }
    p.a.base = (const uint4v *)((size_t)x & ~(size_t)15);
    p.a.x = (const unsigned short *)x;
    const bool two_launches = t.combine == MFR_COMBINE_TWO_LAUNCHES ||
                              (t.combine == MFR_COMBINE_AUTO && grid > kTicketMaxBlocks);
    p.a.partials = s.partials;
    p.a.ticket = two_launches ? nullptr : s.ticket;
    p.a.out = out;

    const hipError_t e = t.kernel == MFR_KERNEL_MFMA
                             ? launch_k<MFR_KERNEL_MFMA>(p, (int)grid, t, stream)
                             : launch_k<MFR_KERNEL_SHFL>(p, (int)grid, t, stream);
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    if (grid > 1 && two_launches) {
        hipLaunchKernelGGL(combine_kernel, dim3(1), dim3(grid > 4096 ? 1024 : 256), 0, stream,
                           (const float *)s.partials, (unsigned int)grid, out);
        const hipError_t e2 = hipGetLastError();
        if (e2 != hipSuccess) return hip_fail(e2, "combine launch");
    }
    return MFR_OK;
}

}  // namespace

extern "C" {

int mfr_sum_f16(const mfr_half *x, size_t n, float *out, hipStream_t stream)
{
    return sum_impl(x, n, out, nullptr, stream);
}

int mfr_sum_f16_tuned(const mfr_half *x, size_t n, float *out, int block_threads, int chain_R,
                      int grid_blocks, int kernel, hipStream_t stream)
{
    // the explicit entry rejects zeros instead of reading them as "default"
    if (block_threads == 0 || chain_R == 0) return MFR_ERR_INVALID_ARG;
    mfr_tuning t;
    memset(&t, 0, sizeof t);
    t.block_threads = block_threads;
    t.chain_R = chain_R;
    t.grid_blocks = grid_blocks;
    t.kernel = kernel;
    return sum_impl(x, n, out, &t, stream);
}

int mfr_sum_f16_ex(const mfr_half *x, size_t n, float *out, const mfr_tuning *t, hipStream_t stream)
{
    return sum_impl(x, n, out, t, stream);
}

int mfr_get_default_tuning(int *block_threads, int *chain_R, int *grid_blocks)
{
    if (block_threads) *block_threads = kDefaultBlock;
    if (chain_R) *chain_R = kDefaultR;
    if (grid_blocks) *grid_blocks = MFR_GRID_AUTO;
    return MFR_OK;
}

long long mfr_grid_for(size_t n, size_t x_addr, const mfr_tuning *tin)
{
    mfr_tuning t;
    if (resolve_tuning(tin, &t) != MFR_OK) return -1;
    if (n == 0) return 1;
    Plan p;
    plan_region(n, x_addr, t, &p);
    int cus = 0;
    if (t.grid_blocks == MFR_GRID_AUTO) {
        int dev = 0;
        DeviceInfo info;
        if (hipGetDevice(&dev) != hipSuccess || device_info(dev, &info) != MFR_OK) return -1;
        cus = info.cus;
    }
    return grid_blocks_for(p, t, cus);
}

int mfr_plan_for(size_t n, size_t x_addr, const mfr_tuning *tin, unsigned long long plan[7])
{
    mfr_tuning t;
    const int st = resolve_tuning(tin, &t);
    if (st != MFR_OK) return st;
    if (!plan || (x_addr & 1u) || n > ((size_t)1 << 60)) return MFR_ERR_INVALID_ARG;
    Plan p;
    plan_region(n, x_addr, t, &p);
    plan[0] = p.a.head;
    plan[1] = p.a.slots;
    plan[2] = p.a.main0;
    plan[3] = p.a.chains;
    plan[4] = p.half ? 32ull : 64ull;
    plan[5] = p.a.epi0;
    plan[6] = p.a.epi1;
    return MFR_OK;
}

const char *mfr_strerror(int status)
{
    switch (status) {
    case MFR_OK: return "success";
    case MFR_ERR_INVALID_ARG: return "invalid argument";
    case MFR_ERR_UNSUPPORTED: return "unsupported device (gfx950 required)";
    case MFR_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

const char *mfr_last_hip_error(void) { return g_hip_error; }

int mfr_version(void) { return 100; }

}  // extern "C"
