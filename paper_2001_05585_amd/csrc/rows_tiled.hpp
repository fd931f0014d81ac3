// Many rows at once: the accumulator columns of one MFMA chain are shared out among rows.
//
// The ones-matrix product of Section 4.1 (eq. MMA1) yields one sum per column
// of the data operand, and the chain C_k = 1 x M_k + C_{k-1} of Section 4.3
// keeps adding tiles into those 16 column sums.  For one long array all 16
// columns belong to the same sum.  Here a tile holds 16 / P rows: P adjacent
// columns (P = 1, 2, 4, 8 or 16) belong to one row, so that after the chain
// along the row a fold over P adjacent lanes (log2 P row-local lane steps, none
// for P = 1) leaves the complete row sum.  P = 16 is one row per tile, P = 1
// sixteen rows per tile.
//
// Lane l = 16 q + j of a wave supplies the 8 k-values 8 q .. 8 q + 7 of column
// j.  With part = j mod P and row_local = j / P, that lane reads the 16-byte
// slot  part + P q + 4 P t  of its row for tile t of the chain: the P lanes of
// a row and one q read P adjacent slots, the four q read four such pieces, so
// one load instruction of the wave covers 64 P contiguous bytes of each of its
// 16 / P rows -- one contiguous KiB when the rows are contiguous and 64 P bytes
// long.
//
// A wave works on GF such tiles ("groups") side by side, i.e. on 16 GF / P
// consecutive rows per iteration, D tiles of each per step; iterations are
// dealt round-robin to the waves of a persistent grid.  The loads of step s+1
// are issued before step s is consumed (two register buffers), so that a wave
// always has loads in flight.
//
// Rows may start at any element (any 16-byte phase, any stride >= cols): a
// row's slots are counted from the 16-byte boundary at or below its first
// element, and slots that are only partly inside the row are masked after loading
// (the bytes outside belong to the gap or to the neighbouring rows, inside the
// array's span).  The few rows at either end whose slots could reach outside
// the span [x, x + span) are left out: the kernel stores rows [row_lo, row_hi)
// only and the host sums the others with the single-row kernel.  Steps in
// which every slot is whole ("plain") run without masks.
#pragma once
#include "mfr_kernels.hpp"

#include <type_traits>

namespace mfr {

struct RowsArgs {
    const char *x;                   // first element of row 0
    unsigned long long span;         // bytes from x to one past the last element of the last row
    unsigned long long rows;
    unsigned long long cols;
    unsigned long long stride_bytes;
    unsigned long long iters;        // ceil(rows / rows per iteration)
    unsigned long long row_lo;       // rows [row_lo, row_hi) are summed here: all their slots lie inside the span
    unsigned long long row_hi;
    unsigned int batches;            // steps per row
    unsigned int plain_lo;           // steps [plain_lo, plain_hi) consist of whole in-row slots only
    unsigned int plain_hi;
    float *out;
};

// Keep elements [lo, hi) of a slot, zero the rest (lo, hi already clamped to 0 .. per_slot).
template <int DT>
__device__ __forceinline__ uint4v mask_slot(uint4v v, int lo, int hi)
{
    const unsigned km = hi > lo ? ((1u << hi) - (1u << lo)) : 0u;     // bit t set: element t stays
    if constexpr (ElemTraits<DT>::per_slot == 8) {
        unsigned m[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned a = (unsigned)(-(int)((km >> (2 * i)) & 1u)), b = (unsigned)(-(int)((km >> (2 * i + 1)) & 1u));
            m[i] = (a & 0xffffu) | (b & 0xffff0000u);
        }
        v.x &= m[0]; v.y &= m[1]; v.z &= m[2]; v.w &= m[3];
    } else {
        v.x &= (unsigned)(-(int)(km & 1u));
        v.y &= (unsigned)(-(int)((km >> 1) & 1u));
        v.z &= (unsigned)(-(int)((km >> 2) & 1u));
        v.w &= (unsigned)(-(int)((km >> 3) & 1u));
    }
    return v;
}

template <int LP>
__device__ __forceinline__ float fold_columns(float v)
{
    if constexpr (LP >= 1) v = dpp_add<0xB1>(v);     // quad_perm [1,0,3,2]
    if constexpr (LP >= 2) v = dpp_add<0x4E>(v);     // quad_perm [2,3,0,1]
    if constexpr (LP >= 3) v = dpp_add<0x141>(v);    // row_half_mirror
    if constexpr (LP >= 4) v = dpp_add<0x140>(v);    // row_mirror
    return v;
}

// DT: element type.  LP: log2 P.  D: tiles of a row per step.  GF: groups side by side.
// ALLPLAIN: the host guarantees that every step is plain (aligned rows of a whole number of steps).
// NT: non-temporal loads and stores.
template <int DT, int LP, int D, int GF, bool ALLPLAIN, bool NT>
__global__ void __launch_bounds__(256) rows_tiled_kernel(const RowsArgs a)
{
    constexpr unsigned P = 1u << LP, RPT = 16u / P;
    constexpr int E = (int)ElemTraits<DT>::per_slot;
    constexpr int LOG_ES = E == 8 ? 1 : 2;
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const unsigned wpb = blockDim.x >> 6;
    const unsigned long long W = (unsigned long long)gridDim.x * wpb;
    const unsigned long long w = (unsigned long long)blockIdx.x * wpb + wave;
    const unsigned j = lane & 15u, q = lane >> 4;
    const unsigned part = j & (P - 1u), row_local = j >> LP;
    const unsigned s_lane = part + P * q;          // this lane's slot inside a tile's 4 P slots per row

    // Row of this lane in group u of iteration `it`: byte offset of its first element from x, and
    // the bytes of its first slot that lie before it.  Rows outside [row_lo, row_hi) are replaced by
    // the nearest row inside (their sums are not stored).
    auto row_of = [&](unsigned long long it, int u, unsigned long long &off, unsigned &ph) {
        unsigned long long r = (it * GF + u) * RPT + row_local;
        r = r < a.row_lo ? a.row_lo : (r < a.row_hi ? r : a.row_hi - 1ull);
        off = r * a.stride_bytes;
        ph = (unsigned)(((unsigned long long)a.x + off) & 15ull);
    };

    // Loads of one step.  Without ALLPLAIN a slot may lie past the row's end: it is replaced by the
    // row's first slot (and masked to zero later).  Plain and masked steps share this code, so that
    // the stream of loads does not depend on control flow.
    auto issue = [&](unsigned long long it, unsigned cb, uint4v (&v)[GF][D], unsigned (&phase)[GF]) {
#pragma unroll
        for (int u = 0; u < GF; ++u) {
            unsigned long long off; unsigned ph;
            row_of(it, u, off, ph);
            phase[u] = ph;                                                       // kept for the masks
            const long long slot0 = (long long)off - (long long)ph;              // first slot of the row, from x
            const long long vend = (long long)(ph >> LOG_ES) + (long long)a.cols;  // row end in slot-relative elements
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const unsigned s = s_lane + 4u * P * ((unsigned)d + (unsigned)D * cb);
                const long long rel = slot0 + 16ll * s;
                if constexpr (ALLPLAIN) {
                    v[u][d] = load_slot<NT>((const uint4v *)(a.x + rel));
                } else {
                    const bool inside = (long long)E * s < vend;
                    v[u][d] = load_slot<NT>((const uint4v *)(a.x + (inside ? rel : slot0)));
                }
            }
        }
    };
    auto is_plain = [&](unsigned cb) { return ALLPLAIN || (cb >= a.plain_lo && cb < a.plain_hi); };

    float4v acc[GF];                                                 // C_0 = 0
#pragma unroll
    for (int u = 0; u < GF; ++u) acc[u] = float4v{0.f, 0.f, 0.f, 0.f};

    auto consume = [&](unsigned long long it, unsigned cb, uint4v (&v)[GF][D], const unsigned (&phase)[GF]) {
        if constexpr (!ALLPLAIN) {
            if (!is_plain(cb)) {
#pragma unroll
                for (int u = 0; u < GF; ++u) {
                    const long long head = (long long)(phase[u] >> LOG_ES), vend = head + (long long)a.cols;
#pragma unroll
                    for (int d = 0; d < D; ++d) {
                        const long long e0 = (long long)E * (s_lane + 4u * P * ((unsigned)d + (unsigned)D * cb));
                        long long lo = head - e0, hi = vend - e0;
                        lo = lo < 0 ? 0 : (lo > E ? E : lo);
                        hi = hi < 0 ? 0 : (hi > E ? E : hi);
                        v[u][d] = mask_slot<DT>(v[u][d], (int)lo, (int)hi);
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < GF; ++u)
#pragma unroll
            for (int d = 0; d < D; ++d) acc[u] = mma_ones<DT>(v[u][d], acc[u]);
        if (cb + 1u == a.batches) {
            // Every lane of a row's P columns holds, after the fold, that row's sum for each group;
            // the lanes with part 0 and q = u mod 4 store group u.
#pragma unroll
            for (int h = 0; h < (GF + 3) / 4; ++h) {
                float val = acc[4 * h].x;
#pragma unroll
                for (int u = 1; u < 4 && 4 * h + u < GF; ++u) val = q == (unsigned)u ? acc[4 * h + u].x : val;
                val = fold_columns<LP>(val);
                const unsigned long long r = (it * GF + 4u * h + q) * RPT + row_local;
                if (part == 0u && 4u * h + q < (unsigned)GF && r >= a.row_lo && r < a.row_hi) {
                    // a store instruction covers 64 / P rows; streaming stores pay only for whole 128-byte lines
                    if constexpr (NT && LP <= 1) __builtin_nontemporal_store(val, a.out + r);
                    else a.out[r] = val;
                }
            }
#pragma unroll
            for (int u = 0; u < GF; ++u) acc[u] = float4v{0.f, 0.f, 0.f, 0.f};
        }
    };

    // Steps (it, cb) of this wave in order; two register buffers alternate.  The loop has one exit,
    // at its end, and its body is straight-line apart from the masks: with an exit in the middle the
    // compiler's bookkeeping of loads in flight falls back to waiting for all of them.
    if (w >= a.iters) return;
    const unsigned long long steps = ((a.iters - w + W - 1ull) / W) * a.batches;     // >= 1
    auto advance = [&](unsigned long long &it, unsigned &cb) {
        if (++cb == a.batches) { cb = 0u; it += W; }
    };
    uint4v v0[GF][D], v1[GF][D];
    unsigned ph0[GF], ph1[GF];
    unsigned long long it0 = w, it1 = w;
    unsigned cb0 = 0u, cb1 = 0u;
    unsigned long long k = 0;                   // step held in v0
    issue(it0, cb0, v0, ph0);
    while (k + 2ull < steps) {
        it1 = it0; cb1 = cb0; advance(it1, cb1);
        issue(it1, cb1, v1, ph1);
        __builtin_amdgcn_sched_barrier(0);
        consume(it0, cb0, v0, ph0);
        it0 = it1; cb0 = cb1; advance(it0, cb0);
        issue(it0, cb0, v0, ph0);
        __builtin_amdgcn_sched_barrier(0);
        consume(it1, cb1, v1, ph1);
        k += 2ull;
    }
    if (k + 1ull < steps) {
        it1 = it0; cb1 = cb0; advance(it1, cb1);
        issue(it1, cb1, v1, ph1);
        __builtin_amdgcn_sched_barrier(0);
        consume(it0, cb0, v0, ph0);
        consume(it1, cb1, v1, ph1);
    } else {
        consume(it0, cb0, v0, ph0);
    }
}

template <int DT, int LP, int D, int GF>
static hipError_t launch_cfg(const RowsArgs &a, unsigned grid, bool all_plain, bool nt, hipStream_t stream)
{
    const dim3 g(grid), b(256);
    if (all_plain) {
        if (nt) hipLaunchKernelGGL((rows_tiled_kernel<DT, LP, D, GF, true, true>), g, b, 0, stream, a);
        else hipLaunchKernelGGL((rows_tiled_kernel<DT, LP, D, GF, true, false>), g, b, 0, stream, a);
    } else {
        if (nt) hipLaunchKernelGGL((rows_tiled_kernel<DT, LP, D, GF, false, true>), g, b, 0, stream, a);
        else hipLaunchKernelGGL((rows_tiled_kernel<DT, LP, D, GF, false, false>), g, b, 0, stream, a);
    }
    return hipGetLastError();
}

// Fills in the kernel arguments and launches the instance for the shape.
template <int DT>
hipError_t launch_rows_tiled_dt(const void *x, unsigned long long rows, unsigned long long cols,
                                unsigned long long row_stride, float *out, const RowsTiledShape &s, unsigned grid,
                                bool nt, hipStream_t stream)
{
    constexpr unsigned esize = 16u / ElemTraits<DT>::per_slot;
    RowsArgs a;
    a.x = (const char *)x;
    a.span = ((rows - 1ull) * row_stride + cols) * esize;
    a.rows = rows;
    a.cols = cols;
    a.stride_bytes = row_stride * esize;
    a.iters = s.iters;
    a.row_lo = s.row_lo;
    a.row_hi = s.row_hi;
    a.batches = s.batches;
    a.plain_lo = s.plain_lo;
    a.plain_hi = s.plain_hi;
    a.out = out;
    const int key = s.log2_p * 100 + s.tiles_per_step * 10 + s.groups;
    switch (key) {
    case 18: return launch_cfg<DT, 0, 1, 8>(a, grid, s.all_plain, nt, stream);
    case 118: return launch_cfg<DT, 1, 1, 8>(a, grid, s.all_plain, nt, stream);
    case 218: return launch_cfg<DT, 2, 1, 8>(a, grid, s.all_plain, nt, stream);
    case 318: return launch_cfg<DT, 3, 1, 8>(a, grid, s.all_plain, nt, stream);
    case 414: return launch_cfg<DT, 4, 1, 4>(a, grid, s.all_plain, nt, stream);
    case 441: return launch_cfg<DT, 4, 4, 1>(a, grid, s.all_plain, nt, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace mfr
