// Device code of libmfreduce (gfx950): the single-pass reduction of paper
// Section 5.2 in three levels.
//   1. every wavefront runs chains of R MFMAs  C_r = 1 x M_r + C_{r-1}
//      (Section 4.3) with an fp32 accumulator, and folds each finished chain
//      to one fp32 partial;
//   2. the waves of a block combine their partials through LDS;
//   3. every block hands its partial to the block with the highest index,
//      which adds them in index order and writes the result, or a second
//      one-block launch does (the paper adds them with float atomics, whose
//      order varies from run to run).
// A conventional kernel (per-lane fp32 accumulation + wave shuffle tree, the
// comparison kernel of Section 5.4) shares levels 2 and 3.
//
// Memory view.  The input is addressed in 16-byte "slots" counted from x
// rounded down to a 16-byte boundary.  Slot 0 may start before x (head
// padding) and the last slot may end after x + n; those two are read
// element-wise under a range check, padding contributes +0 (the border
// handling Section 4.1 leaves to the implementation).  All other slots are
// read with one 128-bit load per lane, 64 lanes = 1 KiB contiguous per load
// instruction = one tile.  Any assignment of elements to matrix positions
// yields the same total, so the layout is chosen for coalescing alone.
//
// Element types: binary16 (the paper's), bfloat16 and binary32.  A tile is one
// 16x16x32 MFMA for the 16-bit types (8 values per lane).  For binary32 (4
// values per lane) the lane first adds its four values in fp32 and one
// 16x16x4 MFMA per tile adds the lanes' sums into the accumulator columns, so
// three of every four additions of that type are vector-ALU additions.
//
// Precision.  Inside a chain everything is fp32, as in the paper: the MFMA
// accumulator, and the fold of its 16 column sums to the chain's fp32 result.
// A wave adds its chains' fp32 results into a binary64 running sum, and the
// block and grid combines stay in binary64 until the one rounding to fp32 per
// block partial and the one of the final result.  The number of dependent fp32
// additions therefore does not grow with the number of chains a wave runs
// (which a caller-chosen small grid can make very large).
#ifndef MFR_KERNELS_HPP
#define MFR_KERNELS_HPP

#include <hip/hip_runtime.h>

#include "mfreduce.h"

namespace mfr {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

constexpr int kMaxWavesPerBlock = 16;

// Type of a wave's running sum over its chains' fp32 results.
#ifdef MFR_WAVE_ACC_F32
typedef float WaveAcc;
#else
typedef double WaveAcc;
#endif

struct SumArgs {
    const uint4v *base;          // slot 0 (of row 0): x rounded down to 16 bytes
    const void *x;               // first element (of row 0)
    unsigned long long n;        // elements per row
    unsigned long long vend;     // head + n: end of the valid range in slot-relative elements
    unsigned long long main0;    // first slot of the unmasked main region
    unsigned long long chains;   // number of full chains in the main region
    unsigned long long epi0;     // border positions [epi0, epi1)
    unsigned long long epi1;
    unsigned long long slots;    // total slots covering [x, x + n)
    unsigned long long row_bytes;  // distance between rows in bytes
    unsigned long long split_chains;  // MFR_KERNEL_SPLIT: chains [0, split_chains) take the MFMA path ...
    unsigned long long split_waves;   // ... on waves [0, split_waves); the rest is conventional
    unsigned int head;           // elements of slot 0 that lie before x
    unsigned int per_row_phase;  // nonzero: the rows of a batched call differ in 16-byte phase; each block then
                                 // derives base, head, vend, main0, chains, epi0, epi1 and slots of its row
                                 // itself (the values above are those of a row that starts on a boundary)
    float *partials;             // two-launch combine: gridDim.x per row, read by combine_kernel
    unsigned int *combine_slots; // single-launch combine: gridDim.x words per row, all zero between calls;
                                 // nullptr = two-launch combine
    float *out;                  // one per row
    unsigned long long rotate_bytes;  // 0, or: row r reads its chains starting r * rotate_bytes further on (rounded to
                                      // whole chains, modulo the row's chains) and wrapping round
    unsigned long long *stamps;  // diagnostic: four wall-clock readings per block (see mfr_sum_f16_stamped); normally nullptr
};

// Slot arithmetic of one array of n elements whose first element lies `head` elements past a
// 16-byte boundary: slot 0 is the (partial) head slot, full slots [main0, main0 + chains *
// chain_slots) form the chains, the border positions [epi0, epi1) take the rest (position `slots`
// stands for the head slot).  Used by the host for a single array and for rows of equal phase,
// and by each block of the kernel for its own row when the phases differ.
__host__ __device__ inline void region_fields(unsigned long long n, unsigned int head, unsigned int per_slot,
                                              unsigned int chain_slots, SumArgs *a)
{
    const unsigned long long vend = (unsigned long long)head + n;
    const unsigned long long slots = (vend + per_slot - 1ull) / per_slot;
    const unsigned long long s0 = head ? 1ull : 0ull;
    const unsigned long long s1 = vend / per_slot;             // slots that end at or before vend
    const unsigned long long full = s1 > s0 ? s1 - s0 : 0ull;
    const unsigned long long chains = full / chain_slots;
    a->head = head;
    a->n = n;
    a->vend = vend;
    a->main0 = s0;
    a->chains = chains;
    a->epi0 = s0 + chains * chain_slots;
    a->epi1 = slots + s0;
    if (a->epi0 > a->epi1) a->epi0 = a->epi1;                  // n smaller than the head slot
    a->slots = slots;
}

struct Plan {
    SumArgs a;
    int threads;                 // launched threads per block (>= 64)
    int waves;                   // waves per block
    bool half;                   // 32-thread geometry
    unsigned long long chains;
    unsigned int dynamic_lds = 0;   // bytes of LDS asked for beyond what the kernel uses: limits the blocks resident per CU
};

template <int DT> struct ElemTraits;
template <> struct ElemTraits<MFR_DTYPE_F16> { static constexpr unsigned per_slot = 8; typedef unsigned short storage; };
template <> struct ElemTraits<MFR_DTYPE_BF16> { static constexpr unsigned per_slot = 8; typedef unsigned short storage; };
template <> struct ElemTraits<MFR_DTYPE_F32> { static constexpr unsigned per_slot = 4; typedef unsigned int storage; };

// ---------------------------------------------------------------- loads ---

// One aligned 16-byte slot.
template <bool NT>
__device__ __forceinline__ uint4v load_slot(const uint4v *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

// Slot q with every element range-checked against [x, x + n).  A slot that
// lies wholly inside is one 128-bit load; a straddling slot is read with
// independent element loads whose indices are clamped into range, so that all
// of them are in flight together, and out-of-range elements are replaced by +0.
// (The level kernel of the recurrence variant reads its groups this way: there a
// value's place in its tile matters.  The single-pass kernels use load_epilogue
// and load_stragglers, which branch around no load.)
template <int DT>
__device__ __forceinline__ uint4v load_slot_guarded(const SumArgs &a, const uint4v *base, const void *x,
                                                    unsigned long long q, bool active)
{
    constexpr unsigned E = ElemTraits<DT>::per_slot;
    typedef typename ElemTraits<DT>::storage storage;
    const unsigned long long v0 = q * E;
    const bool full = active && v0 >= a.head && v0 + E <= a.vend;
    uint4v r = {0u, 0u, 0u, 0u};
    if (full) r = load_slot<false>(base + q);
    if (active && !full) {
        unsigned int h[E];
#pragma unroll
        for (unsigned k = 0; k < E; ++k) {
            const unsigned long long v = v0 + k;
            const bool ok = v >= a.head && v < a.vend;
            const unsigned int t = ((const storage *)x)[ok ? v - a.head : 0ull];   // n >= 1: x[0] is readable
            h[k] = ok ? t : 0u;
        }
        if constexpr (E == 8) {
            r.x = h[0] | (h[1] << 16);
            r.y = h[2] | (h[3] << 16);
            r.z = h[4] | (h[5] << 16);
            r.w = h[6] | (h[7] << 16);
        } else {
            r.x = h[0]; r.y = h[1]; r.z = h[2]; r.w = h[3];
        }
    }
    return r;
}

// A slot of zeros in device memory: where a lane has nothing to load, its load goes here instead of
// being branched around (a branch around a load makes the compiler wait for the loads before it).
static __device__ __align__(16) const unsigned int zero_slot[4] = {0u, 0u, 0u, 0u};

// Border position p -> slot: positions past the last slot stand for slot 0 (the head slot is skipped by
// the main region and picked up here); positions at or past epi1 yield zeros.  Only slots that lie wholly
// inside [x, x + n) are loaded, with one 128-bit load; a slot that straddles either end of the array
// yields zeros here and its elements inside the array come through load_stragglers.  No branch: the loads
// of all border positions of a wave are in flight together.
template <int DT>
__device__ __forceinline__ uint4v load_epilogue(const SumArgs &a, const uint4v *base, const void *x,
                                                unsigned long long p, bool carries)
{
    constexpr unsigned E = ElemTraits<DT>::per_slot;
    (void)x;
    const unsigned long long q = p < a.slots ? p : 0ull, v0 = q * E;
    const bool full = carries && p < a.epi1 && v0 >= a.head && v0 + E <= a.vend;
    // both pointers are named as global memory, or the select between them would be compiled to flat loads
    typedef __attribute__((address_space(1))) const uint4v global_slot;
    const global_slot *from = full ? (const global_slot *)(base + q) : (const global_slot *)zero_slot;
    return *from;
}

// The elements of the array that lie in no wholly valid slot: those before the first slot boundary
// (fewer than a slot, when x is not on a boundary) and those after the last one (fewer than a slot; all
// of the array if it has no whole slot).  Lane k of the first E lanes takes the k-th of the former, lane
// E + k the k-th of the latter, each with one element-wide load at an index clamped into the array; the
// value becomes element 0 of an otherwise empty slot (which position of which tile a value occupies does
// not change the sum).  One load instruction, no branch.
template <int DT>
__device__ __forceinline__ uint4v load_stragglers(const SumArgs &a, const void *x, unsigned lane)
{
    constexpr unsigned E = ElemTraits<DT>::per_slot;
    typedef typename ElemTraits<DT>::storage storage;
    const unsigned long long first_whole = a.head ? 1ull : 0ull, end_whole = a.vend / E;      // whole slots [first_whole, end_whole)
    const unsigned long long front_end = a.vend < first_whole * E ? a.vend : first_whole * E;  // front: [head, front_end)
    const unsigned long long back_begin = (end_whole > first_whole ? end_whole : first_whole) * E;   // back: [back_begin, vend)
    const bool back_lane = lane >= E;
    const unsigned long long v = (back_lane ? back_begin : (unsigned long long)a.head) + (lane & (E - 1u));
    const bool ok = lane < 2u * E && (back_lane ? v < a.vend : v < front_end);
    const unsigned int t = ((const storage *)x)[ok ? v - a.head : 0ull];        // n >= 1: x[0] is readable
    return uint4v{t & (0u - (unsigned int)ok), 0u, 0u, 0u};       // a mask, not a select: the load stays unconditional
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

template <int CTRL>
__device__ __forceinline__ double dpp_add_f64(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, false);
    return v + __hiloint2double(hi, lo);
}

// Sum over each row of 16 lanes in binary64, result in every lane of the row.
__device__ __forceinline__ double row16_sum_f64(double v)
{
    v = dpp_add_f64<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add_f64<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add_f64<0x141>(v);   // row_half_mirror
    v = dpp_add_f64<0x140>(v);   // row_mirror
    return v;
}

// Sum over the 64 lanes in binary64, wave-uniform: DPP within each row of 16 lanes (no trip
// through the LDS crossbar), then the four row sums.
__device__ __forceinline__ double wave64_sum_f64(double v)
{
    v = row16_sum_f64(v);
    double r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        r[k] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 16 * k),
                                __builtin_amdgcn_readlane(__double2loint(v), 16 * k));
    return (r[0] + r[1]) + (r[2] + r[3]);
}

// The same for either running-sum type (the conventional path's per-lane sums).
__device__ __forceinline__ float wave64_sum_acc(float v) { return wave64_sum(v); }
__device__ __forceinline__ double wave64_sum_acc(double v) { return wave64_sum_f64(v); }

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

// Single-launch grid combine: hand-over of block partials through one word each.
//
// A slot is a 32-bit (64-bit for binary64 partials) word of device memory that is zero between
// calls.  A block publishes its partial with ONE device-scope atomic exchange of the value's bits --
// +0.0, the only value whose bits are zero, goes as -0.0, which adds the same -- and is done: it
// waits for nothing.  The block with the highest index of the row takes the other blocks' slots
// with device-scope atomic exchanges against zero until each has returned a non-zero word, and
// adds the values in index order in binary64.  The exchange is a read-modify-write, so it is
// performed where the device keeps its memory coherent (never answered from a cache of the
// reader's own die), and it puts the zero back in the same operation.  Value and "it is there"
// travel in the same word, so no ordering between two memory operations is relied on and no fence
// is needed: an exchange returns either the zero that the previous call left (made visible by the
// kernel boundary) or the one value that this call stored.
//
// Why the reader cannot wait forever: workgroups are dispatched in index order, so when the
// highest-index block of a row runs, every block it waits for has been dispatched or is waiting for
// a compute unit that the reader, a single workgroup, does not hold.  None of them waits for
// anything.  The spin limit below (seconds) only turns a device that stopped making progress into a
// NaN result instead of a hang.
constexpr unsigned int kSpinLimit = 1u << 22;

__device__ __forceinline__ unsigned int slot_bits(float v)
{
    const unsigned int b = __float_as_uint(v);
    return b ? b : 0x80000000u;
}
__device__ __forceinline__ unsigned long long slot_bits(double v)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    return b ? b : 0x8000000000000000ull;
}
__device__ __forceinline__ double slot_value(unsigned int b) { return (double)__uint_as_float(b); }
__device__ __forceinline__ double slot_value(unsigned long long b) { return __longlong_as_double((long long)b); }

template <typename Word, typename Value>
__device__ __forceinline__ void publish_slot(Word *slot, Value v)
{
    // a read-modify-write whose result nobody waits for: performed at the coherence point like the
    // reader's exchange, whatever the write policy of this die's cache
    (void)__hip_atomic_exchange(slot, slot_bits(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// All threads of the reading block: sum of slots[0..count) in binary64, fixed order (thread t takes
// t, t + blockDim, ... in rounds of eight exchanges, then lanes, then waves); every slot is zero
// again afterwards.  Result valid in thread 0.
template <typename Word>
__device__ __forceinline__ double gather_slots(Word *slots, unsigned int count, double *lds)
{
    constexpr int K = 8;
    const unsigned int lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, wpb = (blockDim.x + 63u) >> 6;
    const unsigned int step = blockDim.x;
    double acc = 0.0;
    for (unsigned int base = threadIdx.x; base < count; base += K * step) {
        Word v[K];
#pragma unroll
        for (int k = 0; k < K; ++k) v[k] = 0;
        unsigned int spins = 0;
        for (;;) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const unsigned int i = base + (unsigned)k * step;
                if (i < count && v[k] == 0)
                    v[k] = __hip_atomic_exchange(&slots[i], (Word)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            bool pending = false;
#pragma unroll
            for (int k = 0; k < K; ++k) pending |= (base + (unsigned)k * step < count) && v[k] == 0;
            if (!pending) break;
            if (++spins == kSpinLimit) { acc = __builtin_nan(""); break; }
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const unsigned int i = base + (unsigned)k * step;
            if (i < count) acc += slot_value(v[k]);
        }
    }
    acc = wave64_sum_f64(acc);
    if (lane == 0) lds[wave] = acc;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0)
        for (unsigned int w = 0; w < wpb; ++w) total += lds[w];
    return total;
}

// ------------------------------------------------------ tile consumers ---

// One tile of the chain: C = 1 x M + C  (Section 4.3).  A is the all-ones
// operand, B the data tile; every row of C then holds the 16 column sums, i.e.
// lane l holds column (l mod 16) in each of its 4 accumulator registers.
template <int DT>
__device__ __forceinline__ float4v mma_ones(uint4v tile, float4v c)
{
    if constexpr (DT == MFR_DTYPE_F16) {
        const _Float16 one = (_Float16)1.0f;
        const half8 ones = {one, one, one, one, one, one, one, one};
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, __builtin_bit_cast(half8, tile), c, 0, 0, 0);
    } else if constexpr (DT == MFR_DTYPE_BF16) {
        const __bf16 one = (__bf16)1.0f;
        const bf16x8 ones = {one, one, one, one, one, one, one, one};
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, __builtin_bit_cast(bf16x8, tile), c, 0, 0, 0);
    } else {
        // binary32: B is 4x16, one value per lane.  The lane adds its four values (fp32, as the
        // accumulator would) and one MFMA adds the lanes' sums into the columns: a quarter of the
        // matrix instructions for the same result up to rounding order.
        const float lane_sum = (__uint_as_float(tile.x) + __uint_as_float(tile.y)) + (__uint_as_float(tile.z) + __uint_as_float(tile.w));
        return __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, lane_sum, c, 0, 0, 0);
    }
}

// Chain total from the accumulator: the 16 distinct column sums sit in one
// register across the 16 lanes of a row (all rows and registers are copies),
// so an fp32 row fold replaces the final "x ones" MMA and keeps the chain
// result in fp32 (the accumulator is never rounded to a 16-bit type).
__device__ __forceinline__ float chain_total(float4v c)
{
    return row16_sum(c.x);
}

// Conventional path: fp32 sum of the values of one slot.
template <int DT>
__device__ __forceinline__ float slot_sum_f32(uint4v s)
{
    if constexpr (DT == MFR_DTYPE_F16) {
        const half8 h = __builtin_bit_cast(half8, s);
        return (((float)h[0] + (float)h[1]) + ((float)h[2] + (float)h[3])) +
               (((float)h[4] + (float)h[5]) + ((float)h[6] + (float)h[7]));
    } else if constexpr (DT == MFR_DTYPE_BF16) {
        // bfloat16 is the upper half of a binary32
        const float f0 = __uint_as_float(s.x << 16), f1 = __uint_as_float(s.x & 0xffff0000u);
        const float f2 = __uint_as_float(s.y << 16), f3 = __uint_as_float(s.y & 0xffff0000u);
        const float f4 = __uint_as_float(s.z << 16), f5 = __uint_as_float(s.z & 0xffff0000u);
        const float f6 = __uint_as_float(s.w << 16), f7 = __uint_as_float(s.w & 0xffff0000u);
        return ((f0 + f1) + (f2 + f3)) + ((f4 + f5) + (f6 + f7));
    } else {
        return (__uint_as_float(s.x) + __uint_as_float(s.y)) + (__uint_as_float(s.z) + __uint_as_float(s.w));
    }
}

// Internal kind: MFMA chain whose 16 column sums are handed back unfolded
// (lane l gets column l mod 16), for the binary64 accumulation mode.
constexpr int KIND_MFMA_COLUMNS = 16;

// One chain of R tiles to one fp32 value.  MFMA path: the chain total, uniform
// over the wave.  Conventional path: this lane's share of it.
template <int KERNEL, int DT, int R>
__device__ __forceinline__ float consume_chain(const uint4v (&v)[R])
{
    if constexpr (KERNEL == MFR_KERNEL_MFMA || KERNEL == KIND_MFMA_COLUMNS) {
        float4v acc = {0.f, 0.f, 0.f, 0.f};                 // C_0 = 0
#pragma unroll
        for (int r = 0; r < R; ++r) acc = mma_ones<DT>(v[r], acc);
        if constexpr (KERNEL == KIND_MFMA_COLUMNS) return acc.x;
        else return chain_total(acc);
    } else {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r) s += slot_sum_f32<DT>(v[r]);
        return s;
    }
}

// ------------------------------------------------------------- kernels ---

// The chains c, c + stride, c + 2 stride, ... below c_end of one wave, and (if
// `border`) the border tiles.  KIND is MFR_KERNEL_MFMA (returns the wave's sum
// of chain totals, uniform) or MFR_KERNEL_SHFL (returns this lane's fp32 sum).
template <int KIND, int DT, int R, int U, bool NT, bool HALF, typename Acc = float>
__device__ __forceinline__ Acc stream_chains(const SumArgs &a, const uint4v *base, const void *x, unsigned lane,
                                             unsigned long long c, unsigned long long c_end,
                                             unsigned long long stride, bool border, unsigned long long rot = 0ull)
{
    constexpr unsigned TS = HALF ? 32u : 64u;          // slots per tile
    const bool carries = !HALF || lane < 32u;
    const uint4v zero4 = {0u, 0u, 0u, 0u};
    const uint4v *lane_base = base + a.main0 + (carries ? lane : 0u);
    Acc partial = 0;
    // chain c of the wave's sequence is chain (c + rot) mod chains of the array (rot < chains)
    const unsigned long long wrap = a.chains;
    auto placed = [&](unsigned long long cc) { cc += rot; return cc >= wrap ? cc - wrap : cc; };

    // Border: leftover whole tiles (fewer than R) and leftover whole slots, as tiles in chains of R (at
    // most two chains; positions past the end are all zeros), and one tile of stragglers: the elements
    // of the two slots that straddle the ends of the array.  The loads of the first border chain and of
    // the stragglers are issued early and consumed after the main loop: they go out right after the
    // loads of this wave's first main step, so that their round trip runs in the shadow of that step
    // and the wave that carries the border neither starts nor ends with a round trip of its own.
    uint4v vb[R];
    uint4v vs[1] = {uint4v{0u, 0u, 0u, 0u}};
    // an array made of whole slots has no stragglers (uniform over the block)
    const bool stragglers = a.head != 0u || (a.vend % ElemTraits<DT>::per_slot) != 0ull;
    if (border) {
        auto load_border = [&]() {
#pragma unroll
            for (int r = 0; r < R; ++r)
                vb[r] = load_epilogue<DT>(a, base, x, a.epi0 + (unsigned long long)r * TS + lane, carries);
            if (stragglers) vs[0] = load_stragglers<DT>(a, x, lane);
        };
        bool stepped = false;
        if constexpr (U > 1) {
            if (c + (unsigned long long)(U - 1) * stride < c_end) {
                uint4v v[U][R];
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const uint4v *p = lane_base + (placed(c + (unsigned long long)u * stride) * R + r) * TS;
                        v[u][r] = carries ? load_slot<NT>(p) : zero4;
                    }
                __builtin_amdgcn_sched_barrier(0);
                load_border();
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < U; ++u) partial += (Acc)consume_chain<KIND, DT, R>(v[u]);
                c += (unsigned long long)U * stride;
                stepped = true;
            }
        }
        if (!stepped && c < c_end) {
            uint4v v[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint4v *p = lane_base + (placed(c) * R + r) * TS;
                v[r] = carries ? load_slot<NT>(p) : zero4;
            }
            __builtin_amdgcn_sched_barrier(0);
            load_border();
            __builtin_amdgcn_sched_barrier(0);
            partial += (Acc)consume_chain<KIND, DT, R>(v);
            c += stride;
            stepped = true;
        }
        if (!stepped) load_border();
    }

    if constexpr (U > 1) {
        for (; c + (unsigned long long)(U - 1) * stride < c_end; c += (unsigned long long)U * stride) {
            uint4v v[U][R];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const uint4v *p = lane_base + (placed(c + (unsigned long long)u * stride) * R + r) * TS;
                    v[u][r] = carries ? load_slot<NT>(p) : zero4;
                }
            // all U * R loads are issued before the first is consumed
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < U; ++u) partial += (Acc)consume_chain<KIND, DT, R>(v[u]);
        }
    }
    for (; c < c_end; c += stride) {
        uint4v v[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint4v *p = lane_base + (placed(c) * R + r) * TS;
            v[r] = carries ? load_slot<NT>(p) : zero4;
        }
        __builtin_amdgcn_sched_barrier(0);
        partial += (Acc)consume_chain<KIND, DT, R>(v);
    }

    if (border) {
        if (a.epi0 < a.epi1) partial += (Acc)consume_chain<KIND, DT, R>(vb);
        if (stragglers) partial += (Acc)consume_chain<KIND, DT, 1>(vs);
        for (unsigned long long p0 = a.epi0 + (unsigned long long)R * TS; p0 < a.epi1; p0 += (unsigned long long)R * TS) {
            uint4v v[R];
#pragma unroll
            for (int r = 0; r < R; ++r)
                v[r] = load_epilogue<DT>(a, base, x, p0 + (unsigned long long)r * TS + lane, carries);
            partial += (Acc)consume_chain<KIND, DT, R>(v);
        }
    }
    return partial;
}

// KERNEL: MFR_KERNEL_MFMA, MFR_KERNEL_SHFL or MFR_KERNEL_SPLIT.  DT: element
// type.  R: chain length in tiles.  U: chains in flight.  NT: non-temporal
// loads.  HALF: only lanes 0..31 carry data (the "32-thread block" geometry on
// a wave64 machine), a tile is then 32 slots.  blockIdx.y selects the row of a
// batched call.
//
// MFR_KERNEL_SPLIT (Section 5.3, "split in two"): the first a.split_chains
// chains of the domain go through the MFMA path on the first a.split_waves
// waves, the rest of the domain through the conventional path on the other
// waves, all in the same pass.
template <int KERNEL, int DT, int R, int U, bool NT, bool HALF>
__global__ void __launch_bounds__(1024) sum_kernel(const SumArgs launch_args)
{
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform
    const unsigned wpb = (blockDim.x + 63u) >> 6;
    // The gridDim.x blocks of row blockIdx.y share that row.
    const unsigned long long W = (unsigned long long)gridDim.x * wpb;
    const unsigned long long w = (unsigned long long)blockIdx.x * wpb + wave;

    const unsigned long long stamp_start = launch_args.stamps ? wall_clock64() : 0ull;
    SumArgs a = launch_args;             // as seen by this block's row
    const unsigned long long row = blockIdx.y;
    const char *x = (const char *)a.x + row * a.row_bytes;
    const uint4v *base = (const uint4v *)((const char *)a.base + row * a.row_bytes);
    if (launch_args.per_row_phase) {
        // rows of differing 16-byte phase: the slot arithmetic of this row (all wave-uniform)
        const unsigned int before = (unsigned int)((size_t)x & 15u);
        base = (const uint4v *)(x - before);
        region_fields(launch_args.n, before / (16u / ElemTraits<DT>::per_slot), ElemTraits<DT>::per_slot,
                      (HALF ? 32u : 64u) * (unsigned)R, &a);
        if constexpr (KERNEL == MFR_KERNEL_SPLIT) {
            // the host split the chains of a row that starts on a boundary; this row may have one fewer
            if (launch_args.split_chains >= launch_args.chains || launch_args.split_chains > a.chains)
                a.split_chains = a.chains;
        }
    }

    // staggered rows of a batched call: this row's first chain (uniform over the block)
    unsigned long long rot = 0ull;
    if (launch_args.rotate_bytes != 0ull) {
        constexpr unsigned long long chain_bytes = (HALF ? 512ull : 1024ull) * (unsigned)R;
        rot = ((row * launch_args.rotate_bytes + chain_bytes / 2ull) / chain_bytes) % a.chains;
    }

    // Level 1: the wave's running sum over the fp32 results of its chains.  MFMA path: uniform over
    // the wave.  Conventional path: one running sum per lane, added up across the wave at the end.
    WaveAcc partial;
    if constexpr (KERNEL == MFR_KERNEL_MFMA) {
        partial = stream_chains<MFR_KERNEL_MFMA, DT, R, U, NT, HALF, WaveAcc>(a, base, x, lane, w, a.chains, W, w == W - 1, rot);
    } else if constexpr (KERNEL == MFR_KERNEL_SHFL) {
        partial = wave64_sum_acc(stream_chains<MFR_KERNEL_SHFL, DT, R, U, NT, HALF, WaveAcc>(a, base, x, lane, w, a.chains, W, w == W - 1, rot));
    } else {
        const unsigned long long W1 = a.split_waves, C1 = a.split_chains;
        if (w < W1) {
            partial = stream_chains<MFR_KERNEL_MFMA, DT, R, U, NT, HALF, WaveAcc>(a, base, x, lane, w, C1, W1, w == W - 1, rot);
        } else {
            partial = wave64_sum_acc(stream_chains<MFR_KERNEL_SHFL, DT, R, U, NT, HALF, WaveAcc>(a, base, x, lane, C1 + (w - W1),
                                                                                               a.chains, W - W1, w == W - 1, rot));
        }
    }

    const unsigned long long stamp_streamed = a.stamps ? wall_clock64() : 0ull;

    // Level 2: one value per block from its wave partials, added in wave order, rounded to fp32 once.
    __shared__ WaveAcc wave_partials[kMaxWavesPerBlock];
    __shared__ double wave_partials_f64[kMaxWavesPerBlock];
    if (lane == 0) wave_partials[wave] = partial;
    __syncthreads();
    float block_sum = 0.f;
    if (threadIdx.x == 0) {
        WaveAcc t = wave_partials[0];
        for (unsigned int i = 1; i < wpb; ++i) t += wave_partials[i];
        block_sum = (float)t;
    }

    // Level 3: all block partials of the row to one value, in index order.
    float *out = a.out + row;
    // Diagnostic stamps of block b (row 0 only): [4b] start, [4b+1] the block's last chain consumed (read
    // before the block's waves meet), [4b+2] partial handed over, [4b+3] result stored (0 unless it did)
    auto stamp = [&](bool stored) {
        if (a.stamps && threadIdx.x == 0 && row == 0) {
            unsigned long long *st = a.stamps + 4ull * blockIdx.x;
            const unsigned long long now = wall_clock64();
            st[0] = stamp_start;
            st[1] = stamp_streamed;
            st[2] = stored ? stamp_streamed : now;
            st[3] = stored ? now : 0ull;
        }
    };
    if (gridDim.x == 1) {
        if (threadIdx.x == 0) *out = block_sum;
        stamp(true);
        return;
    }
    if (a.combine_slots == nullptr) {
        // two-launch combine: the partial is picked up by combine_kernel
        if (threadIdx.x == 0) a.partials[row * gridDim.x + blockIdx.x] = block_sum;
        stamp(false);
        return;
    }
    // Single-launch combine: every block but the last publishes its partial and is done; the block
    // with the highest index gathers them, adds its own and writes the result.
    unsigned int *slots = a.combine_slots + row * gridDim.x;
    if (blockIdx.x + 1u != gridDim.x) {
        if (threadIdx.x == 0) publish_slot(&slots[blockIdx.x], block_sum);
        stamp(false);
        return;
    }
    const double others = gather_slots(slots, gridDim.x - 1u, wave_partials_f64);
    if (threadIdx.x == 0) *out = (float)(others + (double)block_sum);
    stamp(true);
}

// ------------------------------------------------------------ launching ---

template <int KERNEL, int DT, int R, int U>
hipError_t launch_ru(const Plan &p, dim3 grid, bool nt, hipStream_t stream)
{
    const dim3 b((unsigned)p.threads);
    if (p.half) {
        if constexpr (DT == MFR_DTYPE_F16 && KERNEL != MFR_KERNEL_SPLIT) {
            if (nt) hipLaunchKernelGGL((sum_kernel<KERNEL, DT, R, U, true, true>), grid, b, p.dynamic_lds, stream, p.a);
            else hipLaunchKernelGGL((sum_kernel<KERNEL, DT, R, U, false, true>), grid, b, p.dynamic_lds, stream, p.a);
        } else {
            return hipErrorInvalidValue;   // the 32-thread geometry exists for the paper's type only
        }
    } else {
        if (nt) hipLaunchKernelGGL((sum_kernel<KERNEL, DT, R, U, true, false>), grid, b, p.dynamic_lds, stream, p.a);
        else hipLaunchKernelGGL((sum_kernel<KERNEL, DT, R, U, false, false>), grid, b, p.dynamic_lds, stream, p.a);
    }
    return hipGetLastError();
}

template <int KERNEL, int DT>
hipError_t launch_k(const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream)
{
    const bool nt = t.nontemporal == 2;
#define MFR_CASE(R_, U_) \
    case (R_) * 16 + (U_): return launch_ru<KERNEL, DT, R_, U_>(p, grid, nt, stream);
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

template <int DT>
hipError_t launch_sum(const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream)
{
    if (t.kernel == MFR_KERNEL_MFMA) return launch_k<MFR_KERNEL_MFMA, DT>(p, grid, t, stream);
    if (t.kernel == MFR_KERNEL_SHFL) return launch_k<MFR_KERNEL_SHFL, DT>(p, grid, t, stream);
    if constexpr (DT == MFR_DTYPE_F16) {
        if (t.kernel == MFR_KERNEL_SPLIT && !p.half) return launch_k<MFR_KERNEL_SPLIT, DT>(p, grid, t, stream);
    }
    return hipErrorInvalidValue;
}

// one translation unit per element type (they compile in parallel)
hipError_t launch_sum_f16(const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream);
hipError_t launch_sum_bf16(const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream);
hipError_t launch_sum_f32(const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream);

// Binary64 accumulation mode (launch_wide.hip): fp16 input, double result.
hipError_t launch_sum_wide(const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream);

// Many rows in one launch, the accumulator columns shared out among rows (rows_tiled.hpp); any
// element type, any alignment, any stride >= cols.  The host fills in the shape.
struct RowsTiledShape {
    int log2_p;                  // P = 2^log2_p adjacent accumulator columns per row; 16 / P rows per tile
    int tiles_per_step;          // D: tiles of a row loaded together
    int groups;                  // GF: tiles (of different rows) side by side
    bool all_plain;              // every step consists of whole in-row slots (cols = a whole number of steps)
    bool tail;                   // all steps plain, and up to 4 P_t more slots of every row go through tail tiles,
    int tail_log2_p;             // in which a row has P_t = 2^tail_log2_p adjacent columns (D == 1)
    bool shift;                  // 16-bit elements: rows at odd element addresses are read from one element earlier
    unsigned long long iters;    // ceil(rows / (GF * 16 / P))
    unsigned long long row_hi;   // rows [0, row_hi) go through this kernel: their slots lie inside the array's
                                 // span; extra blocks of the launch sum the rows after them, a wave per row
    unsigned int batches;        // steps per row
    unsigned int plain_hi;       // steps [0, plain_hi) are plain; at most the last step is not
};
#define MFR_DECLARE_ROWS_TILED(name) \
    hipError_t name(const void *x, unsigned long long rows, unsigned long long cols, unsigned long long row_stride, \
                    float *out, const RowsTiledShape &s, unsigned grid, bool nt, hipStream_t stream);
MFR_DECLARE_ROWS_TILED(launch_rows_tiled_f16)
MFR_DECLARE_ROWS_TILED(launch_rows_tiled_bf16)
MFR_DECLARE_ROWS_TILED(launch_rows_tiled_f32)
#undef MFR_DECLARE_ROWS_TILED

// One level of the recurrence variant (recurrence.hip): a.chains groups of R
// tiles, one binary16 value out per group; final_out (if not null) receives the
// value of group 0 as a float.
hipError_t launch_recurrence_level(const SumArgs &a, int R, unsigned short *level_out, float *final_out,
                                   hipStream_t stream);

}  // namespace mfr

#endif  // MFR_KERNELS_HPP
