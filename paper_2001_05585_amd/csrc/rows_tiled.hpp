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
// A row's slots are counted from its own first element, wherever that lies:
// the 128-bit loads need no more than the element's alignment (the device
// serves unaligned vector loads), so rows of any 16-byte phase and any stride
// >= cols look alike and nothing before a row's start is ever read.  Only the
// last step of a row can hold slots that are partly or wholly past the row's
// end; their position is the same for every row, so each lane prepares, once,
// the byte offsets and the bit masks of its slots in that step (a slot wholly
// past the end is replaced by the row's first slot and masked to zero).  The
// bytes masked away belong to the gap or to the next rows, inside the array's
// span; the few rows at the end whose last slot would reach past the span are
// left out of the tiles -- rows [0, row_hi) go through them, and the blocks
// from main_blocks on sum the others, a wave per row, from element-wide loads
// that stay inside the row (the same MFMA chain over the row, one tile of 64
// slots per step).
//
// Rows that are a whole number of steps and at most 256 bytes more do not pay a masked step for those bytes:
// after the row's plain steps, tail tiles take the rest of all rows of the iteration.  A tail tile gives P_t = 1, 2
// or 4 adjacent columns to a row (a rest of up to 64 P_t bytes) and so holds the rests of 16 / P_t rows: lane
// l = 16 q + j reads slot (j mod P_t) + P_t q of the rest of row j / P_t of the tile.  One more MFMA per tail tile
// (eq. MMA1 again) and a fold over P_t columns leave each row's rest in its columns; the storing lanes fetch it
// across lanes.  An iteration of up to 16 / P_t rows has one tail tile (possibly with unused columns), larger
// iterations a whole number of them.
//
// 16-bit elements, rows that start 2 bytes off a 4-byte boundary: 128-bit loads at such addresses run at three
// quarters of the rate.  The SHIFT instances count such a row's slots from the element before its first one (a
// 4-byte boundary; the other rows' slots stay as they are), drop that element from the row's first slot, and
// let the row end one element later in its last step or tail tile.  The element before row 0 shares the aligned
// 32-bit word of x[0]; its value is discarded like every other masked element's.
#pragma once
#include <type_traits>
#include "mfr_kernels.hpp"

namespace mfr {

struct RowsArgs {
    const char *x;                   // first element of row 0
    unsigned long long rows;
    unsigned long long cols;
    unsigned long long stride_bytes;
    unsigned long long iters;        // ceil(rows / rows per iteration)
    unsigned long long row_hi;       // rows [0, row_hi) are summed here: all their slots lie inside the span
    unsigned int batches;            // steps per row (TAIL: the plain steps; the rest of the row is the tail tile)
    unsigned int plain_hi;           // steps [0, plain_hi) consist of whole in-row slots; plain_hi >= batches - 1
    unsigned int main_blocks;        // blocks [0, main_blocks) run the tiles; the blocks after them take rows [row_hi, rows)
    float *out;
};

// a 16-byte slot at element alignment
typedef uint4v slot_unaligned __attribute__((aligned(2)));

// Rows [row_hi, rows), a wave each.  The row's whole slots (counted from its first element) are read with 128-bit
// loads, four tiles of 64 slots in flight; lanes past the last whole slot read a slot of zeros instead of being
// branched around.  The fewer-than-a-slot elements after them come through one element-wide load, lane k taking
// the k-th, as element 0 of an otherwise empty slot.  All tiles are chained through the ones-matrix MFMA
// (Sections 4.1, 4.3) as everywhere else.  Nothing outside the row is read.
template <int DT>
__device__ __forceinline__ void sum_last_rows(const RowsArgs &a)
{
    constexpr unsigned E = ElemTraits<DT>::per_slot;
    typedef typename ElemTraits<DT>::storage storage;
    typedef __attribute__((address_space(1))) const slot_unaligned global_slot;
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const unsigned long long r = a.row_hi + (unsigned long long)(blockIdx.x - a.main_blocks) * (blockDim.x >> 6) + wave;
    if (r >= a.rows) return;
    const char *row = a.x + r * a.stride_bytes;
    const unsigned long long whole = a.cols / E, rest = a.cols % E;
    // the stragglers first: their round trip runs in the shadow of the tiles
    const bool mine = lane < rest;
    const unsigned int t = ((const storage *)row)[mine ? whole * E + lane : 0ull];        // cols >= 1: row[0] is readable
    float4v acc = {0.f, 0.f, 0.f, 0.f};
    for (unsigned long long s0 = 0; s0 < whole; s0 += 256ull) {
        uint4v v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned long long s = s0 + 64ull * (unsigned)i + lane;
            const global_slot *from = s < whole ? (const global_slot *)(row + 16ull * s) : (const global_slot *)zero_slot;
            v[i] = *from;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = mma_ones<DT>(v[i], acc);
    }
    acc = mma_ones<DT>(uint4v{t & (0u - (unsigned int)mine), 0u, 0u, 0u}, acc);
    const float total = chain_total(acc);
    if (lane == 0u) a.out[r] = total;
}

template <bool NT>
__device__ __forceinline__ uint4v load_slot_at(const char *p)
{
    if constexpr (NT) return __builtin_nontemporal_load((const slot_unaligned *)p);
    else return *(const slot_unaligned *)p;
}

// Bit mask that keeps the first `hi` elements of a slot (0 <= hi <= per_slot).
template <int DT>
__device__ __forceinline__ uint4v keep_first(int hi)
{
    const unsigned km = (1u << hi) - 1u;                               // bit t set: element t stays
    uint4v m;
    if constexpr (ElemTraits<DT>::per_slot == 8) {
        unsigned w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned a = (unsigned)(-(int)((km >> (2 * i)) & 1u)), b = (unsigned)(-(int)((km >> (2 * i + 1)) & 1u));
            w[i] = (a & 0xffffu) | (b & 0xffff0000u);
        }
        m.x = w[0]; m.y = w[1]; m.z = w[2]; m.w = w[3];
    } else {
        m.x = (unsigned)(-(int)(km & 1u));
        m.y = (unsigned)(-(int)((km >> 1) & 1u));
        m.z = (unsigned)(-(int)((km >> 2) & 1u));
        m.w = (unsigned)(-(int)((km >> 3) & 1u));
    }
    return m;
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
// ALLPLAIN: every step consists of whole in-row slots (cols is a multiple of the elements per step).
// NT: non-temporal loads and stores.  LPT: -1, or log2 P_t: every step is plain and up to 4 P_t more slots of
// each row go through tail tiles (D == 1).  SHIFT: rows at odd element addresses are read from one element
// earlier (16-bit types, D == 1, with a masked last step or tail tiles).  STEPS: 0, or the number of steps per row
// (2, 3 or 4, == a.batches): the steps of an iteration are then written out one after the other (of two
// iterations when STEPS is odd, so that the two register buffers come round), and tail tiles are loaded with
// the last step only.
template <int DT, int LP, int D, int GF, bool ALLPLAIN, bool NT, int LPT = -1, bool SHIFT = false, int STEPS = 0>
__global__ void __launch_bounds__(256) rows_tiled_kernel(const RowsArgs a)
{
    static_assert(STEPS == 0 || (STEPS >= 2 && STEPS <= 4), "two to four steps are written out");
    constexpr bool TAIL = LPT >= 0;
    constexpr unsigned P = 1u << LP, RPT = 16u / P;
    constexpr unsigned RPI = (unsigned)GF * RPT;          // rows per iteration
    constexpr unsigned PT = TAIL ? 1u << (TAIL ? LPT : 0) : 1u, RPTT = 16u / PT;       // tail tile: columns per row, rows
    constexpr unsigned NTT = TAIL ? (RPI * PT + 15u) / 16u : 1u;                        // tail tiles per iteration
    static_assert(!TAIL || (ALLPLAIN && D == 1 && LPT <= 2 && (NTT == 1u || RPI * PT == NTT * 16u)),
                  "tail tiles follow plain steps; several of them are all full");
    static_assert(!SHIFT || (ElemTraits<DT>::per_slot == 8 && D == 1 && (TAIL || !ALLPLAIN)),
                  "shifted rows end one element later: they need a masked step or a tail tile");
    constexpr long long E = (long long)ElemTraits<DT>::per_slot;
    if (blockIdx.x >= a.main_blocks) {          // uniform over the block
        sum_last_rows<DT>(a);
        return;
    }
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave = (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const unsigned wpb = blockDim.x >> 6;
    const unsigned long long W = (unsigned long long)a.main_blocks * wpb;
    const unsigned long long w = (unsigned long long)blockIdx.x * wpb + wave;
    const unsigned j = lane & 15u, q = lane >> 4;
    const unsigned part = j & (P - 1u), row_local = j >> LP;
    const unsigned s_lane = part + P * q;          // this lane's slot inside a tile's 4 P slots per row

    // The last step of a row, if it is not plain: byte offset of each of this lane's slots from the
    // row's start (0 for a slot wholly past the end) and the mask of the elements inside the row.
    // SHIFT: the same for a row read from one element earlier (one element more to keep); a slot that such a
    // row needs is loaded for every row (for the others all of it is masked away).
    unsigned long long last_off[D];
    uint4v last_keep[D], last_keep_shifted[D];
    if constexpr (!ALLPLAIN) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const unsigned long long s = s_lane + 4ull * P * ((unsigned)d + (unsigned long long)D * (a.batches - 1u));
            const long long from_here = (long long)a.cols - E * (long long)s;      // elements of the row from this slot on
            const long long left = from_here < 0 ? 0 : (from_here > E ? E : from_here);
            const long long left_shifted = from_here + 1 < 0 ? 0 : (from_here + 1 > E ? E : from_here + 1);
            last_off[d] = (SHIFT ? left_shifted : left) > 0 ? 16ull * s : 0ull;
            last_keep[d] = keep_first<DT>((int)left);
            last_keep_shifted[d] = keep_first<DT>((int)left_shifted);
        }
    }

    // TAIL: this lane's slot in a tail tile is slot (j mod P_t) + P_t q of the rest of row j / P_t of the tile
    // (a lone tail tile can have columns past the iteration's rows: those lanes carry nothing): its byte offset
    // in the row and the mask of the elements inside the row, as for a masked step.
    const unsigned row_t = j / PT;                 // this lane's row in a tail tile
    const bool in_tail = row_t < RPI;              // only a lone tail tile has unused columns
    unsigned long long tail_off = 0ull;
    uint4v tail_keep = {0u, 0u, 0u, 0u}, tail_keep_shifted = {0u, 0u, 0u, 0u};
    if constexpr (TAIL) {
        const unsigned long long s = 4ull * P * a.batches + (j & (PT - 1u)) + PT * q;
        const long long from_here = (long long)a.cols - E * (long long)s;
        const long long left = (from_here < 0 || !in_tail) ? 0 : (from_here > E ? E : from_here);
        const long long left_shifted = (from_here + 1 < 0 || !in_tail) ? 0 : (from_here + 1 > E ? E : from_here + 1);
        tail_off = (SHIFT ? left_shifted : left) > 0 ? 16ull * s : 0ull;
        tail_keep = keep_first<DT>((int)left);
        tail_keep_shifted = keep_first<DT>((int)left_shifted);
    }
    // SHIFT: 1 for a row whose first element lies 2 bytes past a 4-byte boundary (byte offset `off` from x)
    const unsigned x_low = (unsigned)(unsigned long long)a.x;
    auto odd_start = [&](unsigned long long off) { return SHIFT ? (((unsigned)off + x_low) >> 1) & 1u : 0u; };
    auto tail_row_offset = [&](unsigned long long it, unsigned tt) {
        unsigned long long r = it * (unsigned long long)RPI + tt * RPTT + (in_tail ? row_t : 0u);
        r = r < a.row_hi ? r : a.row_hi - 1ull;
        return r * a.stride_bytes;
    };

    // Byte offsets from x of this lane's rows in the GF groups of iteration `it`.  An iteration that
    // lies wholly below row_hi needs one scalar product and an add per group; the last one replaces
    // rows from row_hi on by row row_hi - 1 (their sums are not stored).
    const unsigned long long lane_off = (unsigned long long)row_local * a.stride_bytes;
    auto row_offsets = [&](unsigned long long it, unsigned long long (&off)[GF]) {
        const unsigned long long first = it * (unsigned long long)(GF * RPT);          // wave-uniform
        if (first + GF * RPT <= a.row_hi) {
#pragma unroll
            for (int u = 0; u < GF; ++u) off[u] = (first + (unsigned)u * RPT) * a.stride_bytes + lane_off;
        } else {
#pragma unroll
            for (int u = 0; u < GF; ++u) {
                unsigned long long r = first + (unsigned)u * RPT + row_local;
                r = r < a.row_hi ? r : a.row_hi - 1ull;
                off[u] = r * a.stride_bytes;
            }
        }
    };
    auto is_plain = [&](unsigned cb) { return ALLPLAIN || cb < a.plain_hi; };

    // Loads of one step.  The address of a slot is chosen by a select, not by a branch, so that the
    // stream of loads does not depend on control flow.
    // `shifted` gets bit u set if this lane's row of group u is read from one element earlier, bit 24 + t for its
    // row of tail tile t.
    auto issue = [&](unsigned long long it, unsigned cb, uint4v (&v)[GF][D], uint4v (&vt)[NTT], unsigned &shifted,
                     auto with_tail) {
        const bool plain = is_plain(cb);
        unsigned long long off[GF];
        row_offsets(it, off);
        shifted = 0u;
#pragma unroll
        for (int u = 0; u < GF; ++u) {
            const unsigned odd = odd_start(off[u]);
            shifted |= odd << u;
            const char *row = a.x + off[u] - 2u * odd;
#pragma unroll
            for (int d = 0; d < D; ++d) {
                unsigned long long rel = 16ull * (s_lane + 4ull * P * ((unsigned)d + (unsigned long long)D * cb));
                if constexpr (!ALLPLAIN) rel = plain ? rel : last_off[d];
                v[u][d] = load_slot_at<NT>(row + rel);
            }
        }
        // the tail tiles are loaded with every step (no branch around a load; only the last step uses them),
        // unless the steps are written out and this is known not to be the last
        if constexpr (TAIL && decltype(with_tail)::value) {
#pragma unroll
            for (unsigned tt = 0; tt < NTT; ++tt) {
                const unsigned long long off_t = tail_row_offset(it, tt);
                const unsigned odd = odd_start(off_t);
                shifted |= odd << (24u + tt);
                vt[tt] = load_slot_at<NT>(a.x + off_t - 2u * odd + tail_off);
            }
        }
    };

    float4v acc[GF];                                                 // C_0 = 0
#pragma unroll
    for (int u = 0; u < GF; ++u) acc[u] = float4v{0.f, 0.f, 0.f, 0.f};

    // is_last: -1 = the last step of a row is found by comparing cb; 0 / 1 = known
    auto consume = [&](unsigned long long it, unsigned cb, uint4v (&v)[GF][D], uint4v (&vt)[NTT], unsigned shifted,
                       auto is_last) {
        if constexpr (SHIFT) {
            // a shifted row's first slot begins with the element before the row (a select in every step: a
            // branch here makes the compiler wait for all loads in flight)
            const bool first_slot = cb == 0u && s_lane == 0u;
#pragma unroll
            for (int u = 0; u < GF; ++u) v[u][0].x &= (first_slot && ((shifted >> u) & 1u) != 0u) ? 0xffff0000u : 0xffffffffu;
        }
        if constexpr (!ALLPLAIN) {
            if (!is_plain(cb)) {
#pragma unroll
                for (int u = 0; u < GF; ++u)
#pragma unroll
                    for (int d = 0; d < D; ++d) {
                        if constexpr (SHIFT) v[u][d] &= ((shifted >> u) & 1u) != 0u ? last_keep_shifted[d] : last_keep[d];
                        else v[u][d] &= last_keep[d];
                    }
            }
        }
#pragma unroll
        for (int u = 0; u < GF; ++u)
#pragma unroll
            for (int d = 0; d < D; ++d) acc[u] = mma_ones<DT>(v[u][d], acc[u]);
        constexpr int known_last = decltype(is_last)::value;
        if (known_last == 1 || (known_last < 0 && cb + 1u == a.batches)) {
            float tail_sum[NTT];
            if constexpr (TAIL) {
#pragma unroll
                for (unsigned tt = 0; tt < NTT; ++tt) {
                    if constexpr (SHIFT) vt[tt] &= ((shifted >> (24u + tt)) & 1u) != 0u ? tail_keep_shifted : tail_keep;
                    else vt[tt] &= tail_keep;
                    // columns P_t i .. P_t i + P_t - 1: the rest of row i of tail tile tt
                    tail_sum[tt] = fold_columns<TAIL ? LPT : 0>(mma_ones<DT>(vt[tt], float4v{0.f, 0.f, 0.f, 0.f}).x);
                }
            }
            // Every lane of a row's P columns holds, after the fold, that row's sum for each group;
            // the lanes with part 0 and q = u mod 4 store group u.
#pragma unroll
            for (int h = 0; h < (GF + 3) / 4; ++h) {
                float val = acc[4 * h].x;
#pragma unroll
                for (int u = 1; u < 4 && 4 * h + u < GF; ++u) val = q == (unsigned)u ? acc[4 * h + u].x : val;
                val = fold_columns<LP>(val);
                if constexpr (TAIL) {
                    // the row this lane stores is row (4 h + q) RPT + row_local of the iteration: its rest sits in
                    // tail tile row / (16 / P_t), columns P_t (row mod (16 / P_t)) on (every 16-lane row of the
                    // wave holds a copy)
                    const unsigned row_i = (4u * (unsigned)h + q) * RPT + row_local;
                    const int from = (int)((lane & 48u) | (((row_i % RPTT) * PT) & 15u));
                    float rest = __shfl(tail_sum[0], from, 64);
#pragma unroll
                    for (unsigned tt = 1; tt < NTT; ++tt) {
                        const float other = __shfl(tail_sum[tt], from, 64);
                        rest = row_i / RPTT == tt ? other : rest;
                    }
                    val += rest;
                }
                const unsigned long long r = (it * GF + 4u * h + q) * RPT + row_local;
                if (part == 0u && 4u * h + q < (unsigned)GF && r < a.row_hi) {
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
    uint4v vt0[NTT], vt1[NTT];
#pragma unroll
    for (unsigned tt = 0; tt < NTT; ++tt) vt0[tt] = vt1[tt] = uint4v{0u, 0u, 0u, 0u};
    unsigned sh0 = 0u, sh1 = 0u;
    typedef std::integral_constant<bool, true> tail_too;
    typedef std::integral_constant<bool, false> no_tail;
    typedef std::integral_constant<int, -1> last_by_count;
    typedef std::integral_constant<int, 0> not_last [[maybe_unused]];
    typedef std::integral_constant<int, 1> last [[maybe_unused]];

    if constexpr (STEPS != 0) {
        // The steps of PER iterations written out (a.batches == STEPS): step j of the body belongs to iteration
        // j / STEPS of the body, is step j mod STEPS of its rows and lives in buffer j mod 2; PER * STEPS is even,
        // so every body starts in buffer 0.  The loads of the step after are issued before a step is consumed.
        // Tail tiles travel with a row's last step, in the buffer of that step.
        constexpr int PER = (STEPS % 2 == 0) ? 1 : 2;
        auto step = [&](unsigned long long it, auto j_tag, auto total_tag, bool body_follows) {
            constexpr int j = decltype(j_tag)::value, total = decltype(total_tag)::value;
            constexpr int cb = j % STEPS, nj = j + 1, ncb = nj % STEPS;
            const unsigned long long it_j = it + (unsigned long long)(j / STEPS) * W;
            const unsigned long long it_n = it + (unsigned long long)(nj / STEPS) * W;
            typedef std::integral_constant<bool, ncb == STEPS - 1> next_has_tail;
            typedef std::integral_constant<int, cb == STEPS - 1 ? 1 : 0> this_is_last;
            if constexpr (nj < total) {
                if constexpr (nj % 2 == 0) issue(it_n, (unsigned)ncb, v0, vt0, sh0, next_has_tail());
                else issue(it_n, (unsigned)ncb, v1, vt1, sh1, next_has_tail());
                __builtin_amdgcn_sched_barrier(0);
            } else {
                // the first step of the body after this one (total is even: buffer 0, step 0)
                if (body_follows) {
                    issue(it_n, 0u, v0, vt0, sh0, no_tail());
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if constexpr (j % 2 == 0) consume(it_j, (unsigned)cb, v0, vt0, sh0, this_is_last());
            else consume(it_j, (unsigned)cb, v1, vt1, sh1, this_is_last());
        };
        const unsigned long long n_it = (a.iters - w + W - 1ull) / W;       // >= 1
        unsigned long long it = w, done = 0;
        issue(it, 0u, v0, vt0, sh0, no_tail());
        for (; done + (unsigned)PER < n_it; done += (unsigned)PER, it += (unsigned)PER * W) {
            typedef std::integral_constant<int, PER * STEPS> total;
            step(it, std::integral_constant<int, 0>(), total(), true);
            step(it, std::integral_constant<int, 1>(), total(), true);
            if constexpr (PER * STEPS > 2) step(it, std::integral_constant<int, 2>(), total(), true);
            if constexpr (PER * STEPS > 3) step(it, std::integral_constant<int, 3>(), total(), true);
            if constexpr (PER * STEPS > 4) step(it, std::integral_constant<int, 4>(), total(), true);
            if constexpr (PER * STEPS > 5) step(it, std::integral_constant<int, 5>(), total(), true);
        }
        // what is left: one iteration, or two when STEPS is odd; no step follows the last one
        if (PER == 2 && n_it - done == 2ull) {
            typedef std::integral_constant<int, 2 * STEPS> total;
            step(it, std::integral_constant<int, 0>(), total(), false);
            step(it, std::integral_constant<int, 1>(), total(), false);
            step(it, std::integral_constant<int, 2>(), total(), false);
            step(it, std::integral_constant<int, 3>(), total(), false);
            if constexpr (2 * STEPS > 4) step(it, std::integral_constant<int, 4>(), total(), false);
            if constexpr (2 * STEPS > 5) step(it, std::integral_constant<int, 5>(), total(), false);
        } else {
            typedef std::integral_constant<int, STEPS> total;
            step(it, std::integral_constant<int, 0>(), total(), false);
            step(it, std::integral_constant<int, 1>(), total(), false);
            if constexpr (STEPS > 2) step(it, std::integral_constant<int, 2>(), total(), false);
            if constexpr (STEPS > 3) step(it, std::integral_constant<int, 3>(), total(), false);
        }
        return;
    }

    unsigned long long it0 = w, it1 = w;
    unsigned cb0 = 0u, cb1 = 0u;
    unsigned long long k = 0;                   // step held in v0
    issue(it0, cb0, v0, vt0, sh0, tail_too());
    while (k + 2ull < steps) {
        it1 = it0; cb1 = cb0; advance(it1, cb1);
        issue(it1, cb1, v1, vt1, sh1, tail_too());
        __builtin_amdgcn_sched_barrier(0);
        consume(it0, cb0, v0, vt0, sh0, last_by_count());
        it0 = it1; cb0 = cb1; advance(it0, cb0);
        issue(it0, cb0, v0, vt0, sh0, tail_too());
        __builtin_amdgcn_sched_barrier(0);
        consume(it1, cb1, v1, vt1, sh1, last_by_count());
        k += 2ull;
    }
    if (k + 1ull < steps) {
        it1 = it0; cb1 = cb0; advance(it1, cb1);
        issue(it1, cb1, v1, vt1, sh1, tail_too());
        __builtin_amdgcn_sched_barrier(0);
        consume(it0, cb0, v0, vt0, sh0, last_by_count());
        consume(it1, cb1, v1, vt1, sh1, last_by_count());
    } else {
        consume(it0, cb0, v0, vt0, sh0, last_by_count());
    }
}

template <int DT, int LP, int D, int GF, bool ALLPLAIN, int LPT, bool SHIFT, int STEPS>
static hipError_t launch_steps(const RowsArgs &a, unsigned grid, bool nt, hipStream_t stream)
{
    if constexpr (SHIFT && ElemTraits<DT>::per_slot != 8) {
        return hipErrorInvalidValue;                     // only 16-bit rows can start 2 bytes off a 4-byte boundary
    } else {
        const dim3 g(grid), b(256);
        if (nt) hipLaunchKernelGGL((rows_tiled_kernel<DT, LP, D, GF, ALLPLAIN, true, LPT, SHIFT, STEPS>), g, b, 0, stream, a);
        else hipLaunchKernelGGL((rows_tiled_kernel<DT, LP, D, GF, ALLPLAIN, false, LPT, SHIFT, STEPS>), g, b, 0, stream, a);
        return hipGetLastError();
    }
}

// Rows of two to four 1 KiB steps (P = 16, one tile per step) that end in a masked step or in tail tiles, and rows
// of two or three masked 4 KiB steps (four tiles per step), run the instances with the steps written out
// (2060-byte rows 81 -> 85 %, 2300-byte 82 -> 87 %, 6144-byte 83 -> 88 %, binary32 rows of 10000 bytes 81 -> 88 %).
template <int DT, int LP, int D, int GF, bool ALLPLAIN, int LPT, bool SHIFT>
static hipError_t launch_instance(const RowsArgs &a, unsigned grid, bool nt, hipStream_t stream)
{
    // (rows of whole steps do better in the loop over steps: 2048-byte rows 89 % against 87.5 %; eight groups with
    // tail tiles have a single step)
    if constexpr (LP == 4 && ((D == 1 && (LPT >= 0 ? GF == 4 : !ALLPLAIN)) || (D == 4 && !ALLPLAIN))) {
        switch (a.batches) {
        case 2u: return launch_steps<DT, LP, D, GF, ALLPLAIN, LPT, SHIFT, 2>(a, grid, nt, stream);
        case 3u: return launch_steps<DT, LP, D, GF, ALLPLAIN, LPT, SHIFT, 3>(a, grid, nt, stream);
        case 4u:
            if constexpr (D == 1) return launch_steps<DT, LP, D, GF, ALLPLAIN, LPT, SHIFT, 4>(a, grid, nt, stream);
            break;          // four steps of four tiles: no gain (14000-byte rows 88 % against 85 %)
        default: break;
        }
    }
    return launch_steps<DT, LP, D, GF, ALLPLAIN, LPT, SHIFT, 0>(a, grid, nt, stream);
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
    a.rows = rows;
    a.cols = cols;
    a.stride_bytes = row_stride * esize;
    a.iters = s.iters;
    a.row_hi = s.row_hi;
    a.batches = s.batches;
    a.plain_hi = s.plain_hi;
    a.main_blocks = grid;
    a.out = out;
    // rows whose last slot would reach past the array: four to a block, after the blocks of the tiles
    if (s.row_hi < rows) grid += (unsigned)((rows - s.row_hi + 3ull) / 4ull);
    // The instances are those the host's choice of shape can ask for: eight groups for 64- and 128-byte steps
    // and for masked steps, four for unmasked steps of 256 bytes and more and for rows of several 1 KiB steps.
    const int key = s.log2_p * 100 + s.tiles_per_step * 10 + s.groups;
    if (s.tail) {
        if (!s.all_plain || s.tail_log2_p < 0 || s.tail_log2_p > 2) return hipErrorInvalidValue;
        const int tkey = key * 10 + s.tail_log2_p;
        if (s.shift) {
            switch (tkey) {
            case 2140: return launch_instance<DT, 2, 1, 4, true, 0, true>(a, grid, nt, stream);
            case 3180: return launch_instance<DT, 3, 1, 8, true, 0, true>(a, grid, nt, stream);
            case 3181: return launch_instance<DT, 3, 1, 8, true, 1, true>(a, grid, nt, stream);
            case 3182: return launch_instance<DT, 3, 1, 8, true, 2, true>(a, grid, nt, stream);
            case 4140: return launch_instance<DT, 4, 1, 4, true, 0, true>(a, grid, nt, stream);
            case 4141: return launch_instance<DT, 4, 1, 4, true, 1, true>(a, grid, nt, stream);
            case 4142: return launch_instance<DT, 4, 1, 4, true, 2, true>(a, grid, nt, stream);
            case 4180: return launch_instance<DT, 4, 1, 8, true, 0, true>(a, grid, nt, stream);
            case 4181: return launch_instance<DT, 4, 1, 8, true, 1, true>(a, grid, nt, stream);
            case 4182: return launch_instance<DT, 4, 1, 8, true, 2, true>(a, grid, nt, stream);
            default: return hipErrorInvalidValue;
            }
        }
        switch (tkey) {
        case 3180: return launch_instance<DT, 3, 1, 8, true, 0, false>(a, grid, nt, stream);
        case 3181: return launch_instance<DT, 3, 1, 8, true, 1, false>(a, grid, nt, stream);
        case 3182: return launch_instance<DT, 3, 1, 8, true, 2, false>(a, grid, nt, stream);
        case 4140: return launch_instance<DT, 4, 1, 4, true, 0, false>(a, grid, nt, stream);
        case 4141: return launch_instance<DT, 4, 1, 4, true, 1, false>(a, grid, nt, stream);
        case 4142: return launch_instance<DT, 4, 1, 4, true, 2, false>(a, grid, nt, stream);
        case 4180: return launch_instance<DT, 4, 1, 8, true, 0, false>(a, grid, nt, stream);
        case 4181: return launch_instance<DT, 4, 1, 8, true, 1, false>(a, grid, nt, stream);
        case 4182: return launch_instance<DT, 4, 1, 8, true, 2, false>(a, grid, nt, stream);
        default: return hipErrorInvalidValue;
        }
    }
    if (s.shift) {
        if (s.all_plain) return hipErrorInvalidValue;
        switch (key) {
        case 18: return launch_instance<DT, 0, 1, 8, false, -1, true>(a, grid, nt, stream);
        case 118: return launch_instance<DT, 1, 1, 8, false, -1, true>(a, grid, nt, stream);
        case 218: return launch_instance<DT, 2, 1, 8, false, -1, true>(a, grid, nt, stream);
        case 318: return launch_instance<DT, 3, 1, 8, false, -1, true>(a, grid, nt, stream);
        case 414: return launch_instance<DT, 4, 1, 4, false, -1, true>(a, grid, nt, stream);
        case 418: return launch_instance<DT, 4, 1, 8, false, -1, true>(a, grid, nt, stream);
        default: return hipErrorInvalidValue;
        }
    }
    if (s.all_plain) {
        switch (key) {
        case 18: return launch_instance<DT, 0, 1, 8, true, -1, false>(a, grid, nt, stream);
        case 118: return launch_instance<DT, 1, 1, 8, true, -1, false>(a, grid, nt, stream);
        case 214: return launch_instance<DT, 2, 1, 4, true, -1, false>(a, grid, nt, stream);
        case 314: return launch_instance<DT, 3, 1, 4, true, -1, false>(a, grid, nt, stream);
        case 414: return launch_instance<DT, 4, 1, 4, true, -1, false>(a, grid, nt, stream);
        case 441: return launch_instance<DT, 4, 4, 1, true, -1, false>(a, grid, nt, stream);
        default: return hipErrorInvalidValue;
        }
    }
    switch (key) {
    case 18: return launch_instance<DT, 0, 1, 8, false, -1, false>(a, grid, nt, stream);
    case 118: return launch_instance<DT, 1, 1, 8, false, -1, false>(a, grid, nt, stream);
    case 218: return launch_instance<DT, 2, 1, 8, false, -1, false>(a, grid, nt, stream);
    case 318: return launch_instance<DT, 3, 1, 8, false, -1, false>(a, grid, nt, stream);
    case 414: return launch_instance<DT, 4, 1, 4, false, -1, false>(a, grid, nt, stream);
    case 418: return launch_instance<DT, 4, 1, 8, false, -1, false>(a, grid, nt, stream);
    case 441: return launch_instance<DT, 4, 4, 1, false, -1, false>(a, grid, nt, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace mfr
