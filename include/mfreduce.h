/*
 * libmfreduce -- arithmetic reduction of n fp16 numbers to one fp32 on MI355X
 * (gfx950), C ABI.
 *
 * The operation is R(X) = sum_{i=1..n} x_i (paper Section 4, the equation that
 * defines the arithmetic reduction), computed with the single-pass variant of
 * the paper (Section 5.2): every wavefront runs chains of R matrix
 * multiply-accumulates C_r = 1 x M_r + C_{r-1} against an all-ones matrix
 * (Section 4.3), each chain's result is kept as an fp32 partial, wave partials
 * are combined per block, and all block partials are reduced to one fp32.
 *
 * All pointers named "device" must be dereferenceable by kernels on the
 * current HIP device.  No function takes ownership of any pointer.  Every
 * function returns an mfr_status; none throws, prints or exits.  Arguments
 * are validated before the first HIP call, so invalid-argument errors are
 * reported identically on a machine without a GPU.
 */
#ifndef MFREDUCE_H
#define MFREDUCE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* HIP's stream handle; declared here so that callers need no HIP headers. */
typedef struct ihipStream_t *hipStream_t;

/* IEEE 754 binary16 storage (bit-identical to _Float16 / __half). */
typedef uint16_t mfr_half;

typedef enum mfr_status {
    MFR_OK = 0,
    MFR_ERR_INVALID_ARG = 1, /* null pointer, misaligned x, bad block / R / grid / kernel */
    MFR_ERR_UNSUPPORTED = 2, /* current device is not gfx950 */
    MFR_ERR_HIP = 3,         /* a HIP runtime call failed; text via mfr_last_hip_error() */
    MFR_ERR_SCRATCH_LIMIT = 4 /* mfr_sum_f16_noalloc only: the grid needs more scratch than the fixed region holds */
} mfr_status;

/* Element types.  binary16 is the paper's; the other two run the same kernels. */
enum {
    MFR_DTYPE_F16 = 0,  /* IEEE binary16: v_mfma_f32_16x16x32_f16, 8 values per lane per tile */
    MFR_DTYPE_BF16 = 1, /* bfloat16: v_mfma_f32_16x16x32_bf16 */
    MFR_DTYPE_F32 = 2   /* IEEE binary32: 4 values per lane per tile, added in the lane (fp32), then one
                           v_mfma_f32_16x16x4_f32 adds the lanes' sums into the accumulator columns */
};

/* Which kernel computes the block partials. */
enum {
    MFR_KERNEL_MFMA = 0, /* ones-matrix MFMA chains (Sections 4.1, 4.3, 5.2) */
    MFR_KERNEL_SHFL = 1, /* conventional fp32 per-lane accumulate + wave shuffle tree:
                            the comparison kernel of Section 5.4 */
    MFR_KERNEL_SPLIT = 2 /* "split in two" (Section 5.3): a fraction of the domain through the MFMA
                            chains and the rest through the conventional path, in one pass, on
                            disjoint sets of waves.  binary16 only, block_threads >= 64 */
};

/* grid_blocks special values */
enum {
    MFR_GRID_AUTO = 0,       /* persistent grid sized to the device */
    MFR_GRID_ONE_CHAIN = -1  /* the paper's geometry: exactly one chain per wavefront,
                                grid sized to n (Algorithm 2's offset; Section 5.2) */
};

/* How the block partials become one value (Section 5.2 uses float atomics on
 * one location; both modes here add them in index order instead). */
enum {
    MFR_COMBINE_AUTO = 0,          /* single launch for grids up to 2048 blocks, else two */
    MFR_COMBINE_SINGLE_LAUNCH = 1, /* the block with the highest index gathers and adds the partials
                                      (grids above 65536 blocks still use two launches) */
    MFR_COMBINE_TWO_LAUNCHES = 2   /* a second one-block kernel adds the partials */
};

/* Full tuning record for mfr_sum_f16_ex.  Zero in any field selects the
 * library default for that field. */
typedef struct mfr_tuning {
    int block_threads;    /* 32, 64, 128, 256, 512 or 1024.  32 runs as one wave64 whose upper
                             32 lanes contribute zeros (gfx950 has no 32-wide wavefront) */
    int chain_R;          /* 1..8.  MFMA kernel: MFMAs accumulated into one accumulator tile
                             from zero before it is folded to an fp32 partial (the paper's R).
                             SHFL kernel: 16-byte loads per lane accumulated per group.
                             Default: 3 (MFMA, SPLIT; 7 for binary32 input), 6 (SHFL); but a
                             single array of more than 96 KiB and at most 256 MiB for which
                             block_threads, chain_R and chains_in_flight are all left to the
                             library gets 128-thread blocks and one chain of 8 */
    int grid_blocks;      /* MFR_GRID_AUTO, MFR_GRID_ONE_CHAIN, or an explicit count >= 1 */
    int kernel;           /* MFR_KERNEL_MFMA, MFR_KERNEL_SHFL or MFR_KERNEL_SPLIT */
    int chains_in_flight; /* 1, 2, 3, 4, 6 or 8 independent chains whose loads are issued before
                             any is consumed (memory-level parallelism); chain_R *
                             chains_in_flight must not exceed 16.  Default: the count that brings
                             chain_R * chains_in_flight closest to 6 tiles (6 KiB of loads per wave, the
                             measured optimum), the larger count on a tie: 6, 3, 2, 2, 1, 1, 1, 1 for
                             chain_R = 1..8 */
    int nontemporal;      /* 0 = library default (plain loads for inputs up to 32 MiB, which may be
                             resident in the L2s; non-temporal loads beyond), 1 = plain, 2 = non-temporal */
    int combine;          /* MFR_COMBINE_* */
    int split_permille;   /* MFR_KERNEL_SPLIT only: thousandths of the domain (and of the waves) that
                             take the MFMA path, 0..1000 (Section 5.3's fraction f); rounded to whole
                             chains and whole waves */
} mfr_tuning;

/*
 * Sum of x[0..n) (paper Section 4: R(X) = sum x_i; Section 5.2 single pass).
 *
 *   x       device pointer to n binary16 values, 2-byte aligned (16-byte
 *           alignment is NOT required), read-only, never modified.
 *   n       element count; n == 0 writes 0.0f.  64-bit sizes are honoured.
 *   out     device pointer to one float; written once, in stream order.
 *   stream  HIP stream to enqueue on (0 = the null stream).
 *
 * Asynchronous: returns after enqueueing; synchronise the stream before
 * reading *out.  Same (x contents, n, tuning, device) => bit-identical *out:
 * block partials are combined in index order, never with float atomics.
 * Precision: every chain is accumulated and folded in fp32 (32 chain_R + 4
 * dependent additions); the chains of a wave, the waves of a block and the
 * blocks of the grid are added in binary64, with one rounding to fp32 per block
 * partial and one for the result, so the error bound does not depend on how
 * many chains a wave runs (i.e. not on grid_blocks).  The conventional kernel
 * adds the 8 * chain_R values of a lane's group in fp32 and is otherwise alike.
 * IEEE special values propagate (NaN in => NaN; +Inf and -Inf => NaN);
 * subnormal inputs contribute their value (not flushed), for every type.
 * Scratch (one word per block for the grid combine) is owned by the library, one per
 * (device, stream), allocated on first use and kept until mfr_release_scratch
 * or unload; calls on different streams may overlap, calls on one stream
 * serialise on the device.  Host threads may share a stream: the launches of
 * one call are enqueued under a per-stream mutex, so they stay together.  A
 * call whose
 * grid needs more scratch than its stream holds calls hipMalloc for a buffer
 * of at least twice the size; the smaller buffer is kept, not freed, because
 * work that was enqueued or captured earlier still refers to it.  Calls with a
 * grid no larger than before allocate nothing, only launch kernels (no memset
 * nodes), and can therefore be captured into a HIP graph and replayed.
 * A captured call keeps the scratch addresses of the stream it was captured
 * on: replays of such a graph must not overlap with each other or with other
 * calls on that stream, and that stream's scratch must not be released while
 * the graph is in use.
 * With library defaults an array of at most 32 chains (49152 binary16 values)
 * is summed by a single block, which needs no scratch at all.
 */
int mfr_sum_f16(const mfr_half *x, size_t n, float *out, hipStream_t stream);

/*
 * Same sum with caller-chosen geometry (the block size B and chain length R
 * explored in Section 5.2's configuration experiment).  chains_in_flight and
 * the load policy take the library defaults for the given R.
 */
int mfr_sum_f16_tuned(const mfr_half *x, size_t n, float *out,
                      int block_threads, int chain_R, int grid_blocks, int kernel,
                      hipStream_t stream);

/* Same sum with every knob explicit; t == NULL means all defaults. */
int mfr_sum_f16_ex(const mfr_half *x, size_t n, float *out,
                   const mfr_tuning *t, hipStream_t stream);

/*
 * mfr_sum_f16_ex for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same result,
 * bit for bit, as mfr_sum_f16_ex with the same arguments, but the block
 * partials and combine slots live in a fixed 64 KiB array in device memory
 * that is part of the library's code object (every GPU the library runs on
 * holds its own copy from load to process exit), so the call never calls
 * hipMalloc, hipFree or any allocating routine, on any call, the first
 * included.
 *   Limit: grids of at most 8192 blocks; a
 *   tuning that asks for more -- MFR_GRID_ONE_CHAIN on a long input, a large
 *   explicit grid_blocks -- returns MFR_ERR_SCRATCH_LIMIT and enqueues
 *   nothing.  The library defaults (t == NULL) need 256 partials at most.
 *   All calls of this entry point on one GPU share that array, whatever their
 *   stream: calls that overlap in time on one GPU race on it and give wrong
 *   results; calls on one stream, or otherwise ordered, are safe.  The array
 *   needs no clearing: partials are written before they are read within a
 *   call, and every combine slot is back at zero when a call completes.
 */
int mfr_sum_f16_noalloc(const mfr_half *x, size_t n, float *out, const mfr_tuning *t, hipStream_t stream);

/*
 * Diagnostic form of mfr_sum_f16_ex: the same call (Section 5.2's single pass),
 * which also records when each block started, finished its chains, handed its
 * partial over and (the block that does) stored the result, so that the time
 * of a call can be split into start-up, streaming and combine.
 *   stamps      device pointer to stamps_len 64-bit words, stamps_len >= 4 *
 *               mfr_grid_for(n, x, t); block b writes stamps[4b .. 4b+3]:
 *               start, last chain consumed, partial handed over, result stored
 *               (0 for the blocks that do not store it), in ticks of the
 *               device's constant-rate wall clock (mfr_wall_clock_khz)
 * The readings themselves cost a few hundred nanoseconds per call.
 */
int mfr_sum_f16_stamped(const mfr_half *x, size_t n, float *out, const mfr_tuning *t, unsigned long long *stamps,
                        size_t stamps_len, hipStream_t stream);
/* Rate of that clock on the current device, in kHz. */
int mfr_wall_clock_khz(int *khz);

/*
 * The same reduction (Section 4: R(X) = sum x_i, Section 5.2 single pass) for
 * other element types; x must be aligned to its element size.  block_threads
 * == 32 is accepted for binary16 only.  chain_R counts tiles (1 KiB loads per
 * wave) for every type.
 */
int mfr_sum_bf16(const uint16_t *x, size_t n, float *out, hipStream_t stream);
int mfr_sum_f32(const float *x, size_t n, float *out, hipStream_t stream);
int mfr_sum_ex(const void *x, int dtype, size_t n, float *out, const mfr_tuning *t, hipStream_t stream);

/*
 * Batched form: out[r] = sum of x[r * row_stride + c], c in [0, cols), for r in
 * [0, rows) -- one reduction R(X_r) (Section 4) per row through the same
 * ones-matrix chains (Sections 4.1, 4.3).
 *   x           device pointer, aligned to the element size (no more)
 *   row_stride  distance between rows in elements, >= cols when rows > 1; any
 *               value, the rows need not share a 16-byte phase; the whole span
 *               (rows - 1) * row_stride + cols must be below 2^60 elements
 *   out         device pointer to rows floats
 * rows == 0 does nothing; cols == 0 writes zeros.
 * With t == NULL the library picks the kernel: many rows go through one launch
 * in which the 16 accumulator columns of a chain are shared out among rows
 * (mfr_rows_plan shows the shape); few rows, rows of 16 KiB or more, and rows
 * of a 16-bit type of 4 KiB or more that start 2 bytes off a 4-byte boundary
 * get a grid of blocks (or one block) each; of fewer rows than four per
 * compute unit (eight, for rows of 64 KiB and more), row r then starts r * s
 * bytes further on (rounded to whole chains) and wraps round, s being what
 * the row pitch lacks to a multiple of 1 MiB, so that the rows are read, at
 * any one time, at addresses a multiple of 1 MiB apart, which the memory
 * channels take evenly
 * (which chains a wave adds, hence the rounding of out[r], then depends on r
 * and on the pitch; the same call still gives the same bits).
 * That first kernel loads 16-byte slots counted from each row's first element
 * and masks what lies past the row's end, so bytes after a row (in the gap or
 * in the next rows, inside [x, x + ((rows - 1) * row_stride + cols) * element
 * size)) may be read; nothing outside that span is (the last rows, whose final
 * slot would reach past it, are read element by element by extra blocks of the
 * same launch), with one exception: a row
 * of a 16-bit type that starts 2 bytes off a 4-byte boundary is read from that
 * boundary, and its slots are counted from there (the element before the row
 * is discarded).  For row 0 that element lies before x, in the aligned 32-bit
 * word that also holds x[0].
 * With explicit tuning every row is reduced exactly as a single call would
 * (Section 5.2), grid_blocks counting blocks per row and MFR_GRID_AUTO dividing
 * the persistent grid among the rows (rounded down), all rows in one launch (up
 * to 65535 rows per launch).  Every row is read in aligned 16-byte slots, its
 * first and last partial slot element by element, whatever its 16-byte phase;
 * nothing outside a row is read.
 */
int mfr_sum_rows_ex(const void *x, int dtype, size_t rows, size_t cols, size_t row_stride, float *out,
                    const mfr_tuning *t, hipStream_t stream);
int mfr_sum_f16_rows(const mfr_half *x, size_t rows, size_t cols, size_t row_stride, float *out,
                     hipStream_t stream);

/*
 * Higher-accuracy mode of the single-pass sum.  The chains of chain_R MFMAs
 * keep fp32 accumulators as in Section 4.3, but every step after a chain --
 * the running sum per lane, the wave, block and grid combines -- is carried in
 * binary64 and the result is returned as a double.  The remaining error is
 * that of the 32 * chain_R fp32 additions inside one accumulator column, so it
 * does not grow with n: |result - sum| <= (32 chain_R + 4) 2^-24 sum|x_i| in the
 * worst case, far less in practice; integer-valued inputs are summed exactly
 * up to 2^53.  (Sections 2.2 and 5.4 discuss the precision of fp32 partials.)
 *   out   device pointer to one double, 8-byte aligned.
 *   t     as for mfr_sum_f16_ex; kernel must be MFR_KERNEL_MFMA, block_threads
 *         >= 64, chain_R 1..8 (default 1, with six chains in flight).
 */
int mfr_sum_f16_f64(const mfr_half *x, size_t n, double *out, hipStream_t stream);
int mfr_sum_f16_f64_ex(const mfr_half *x, size_t n, double *out, const mfr_tuning *t, hipStream_t stream);

/*
 * Variant #1 of the paper, "recurrence" (Section 5.1; Algorithms 1 and 2 with
 * chains of chain_R MMAs, Section 4.3), as published: each level reduces every
 * group of chain_R * 512 values to one value STORED AS binary16 (the 16 column
 * sums of the chain are rounded to binary16, a last MMA adds them, the group
 * total is rounded to binary16), and levels are relaunched until one value is
 * left.  Provided to reproduce the behaviour Section 5.4 reports: the result
 * carries binary16 rounding at every level and becomes +-Inf as soon as a group
 * sum passes 65504.  Use mfr_sum_f16 for an accurate sum.
 *   x, n, out, stream  as for mfr_sum_f16 (x is not modified: the levels live in
 *                      library scratch); chain_R in 1..8.
 * Groups are counted from x rounded down to 16 bytes (leading padding is zero).
 */
int mfr_sum_f16_recurrence(const mfr_half *x, size_t n, float *out, int chain_R, hipStream_t stream);

/*
 * The geometry mfr_sum_f16 uses for inputs of more than 256 MiB (smaller ones:
 * see mfr_tuning.chain_R).  Any pointer may be NULL.
 * The environment variables MFR_BLOCK (32 .. 1024, a power of two) and MFR_R
 * (1 .. 8), read once per process, replace the built-in default block size and
 * chain length wherever a call leaves them to the library (the B and R of
 * Section 5.2 without recompiling the caller); if either is set to anything
 * else, this call and every call that relies on the default return
 * MFR_ERR_INVALID_ARG.  block 32 is for binary16 only.
 */
int mfr_get_default_tuning(int *block_threads, int *chain_R, int *grid_blocks);

/* Number of blocks a call with this tuning would launch for n elements whose
 * first element has byte address x_addr (only its low 4 bits matter); -1 on
 * invalid tuning.  Touches the device only for MFR_GRID_AUTO. */
long long mfr_grid_for(size_t n, size_t x_addr, const mfr_tuning *t);

/*
 * How a call would split the input (inspection only, no device access):
 *   plan[0] head elements of the first 16-byte slot that lie before x (0..7)
 *   plan[1] total 16-byte slots covering [x, x + n)
 *   plan[2] first slot of the unmasked main region
 *   plan[3] full chains in the main region (each chain_R tiles)
 *   plan[4] slots per tile (64, or 32 for block_threads == 32)
 *   plan[5], plan[6] border positions [begin, end): position p stands for slot
 *           p, or for slot 0 when p >= plan[1]; a slot that lies wholly inside
 *           the array is read with one 128-bit load, the elements of the two
 *           slots that straddle its ends one by one, range-checked
 * The main region reads slots [plan[2], plan[2] + plan[3] * chain_R * plan[4])
 * with unchecked 128-bit loads, so all of them must lie inside [x, x + n).
 */
int mfr_plan_for(size_t n, size_t x_addr, const mfr_tuning *t, unsigned long long plan[7]);
/* The same for any element type (a slot holds 8 16-bit or 4 32-bit values). */
int mfr_plan_ex(size_t n, size_t x_addr, int dtype, const mfr_tuning *t, unsigned long long plan[7]);

/*
 * Shape of the many-rows kernel that mfr_sum_rows_ex(..., t == NULL, ...) would
 * launch on a device with `cus` compute units (inspection only, no device
 * access).  Returns 1 and fills plan[] if that kernel is chosen, 0 if the rows
 * go to the per-row kernels instead, negative status on invalid arguments.
 *   plan[0]  P: adjacent accumulator columns per row (1, 2, 4, 8, 16); a tile holds 16 / P rows
 *   plan[1]  D: tiles of a row per step        plan[2]  GF: tiles side by side
 *   plan[3]  iterations (each GF * 16 / P consecutive rows)
 *   plan[4]  steps per row; step c, tile d gives lane l = 16 q + j the slot
 *            (j mod P) + P q + 4 P (d + D c) of row j / P of its tile, slots being
 *            counted from the row's own first element (128-bit loads at element
 *            alignment)
 *   plan[5], plan[6]  steps [begin, end) made of whole in-row slots only; begin is 0
 *            and at most the last step is left out: its slots are masked, and a
 *            slot wholly past the row's end is replaced by the row's first slot
 *   plan[7], plan[8]  rows [begin, end) that this kernel sums (begin is 0): no slot
 *            of theirs reaches past the array's span; the few rows after them are
 *            summed a wave each, from element-wide loads inside the row, by one
 *            further block per four rows in the same launch (in a tile that holds
 *            rows of both kinds they are replaced by row end - 1, and not stored)
 *   plan[9]  1 if every step is unmasked    plan[10] blocks of 256 threads that run the tiles (one per compute
 *            unit, two for some shapes)
 *   plan[11] bit 0: the rows end in tail tiles: plan[4] then counts the plain steps only (plan[9] is 1), and
 *            the at most 4 P_t slots of each row after them (P_t = 2^(plan[11] >> 2) = 1, 2 or 4) are read as
 *            tiles of 16 / P_t rows each, ceil(GF * P_t / P) of them per iteration: in tail tile t, lane
 *            l = 16 q + j reads slot 4 P plan[4] + (j mod P_t) + P_t q of row t * 16 / P_t + j / P_t of the
 *            iteration (lanes whose row lies past the iteration's GF * 16 / P rows read nothing of their
 *            own; masked and substituted like a masked step's slots).
 *            bit 1 (16-bit types, when some row starts 2 bytes off a 4-byte boundary): such a row's slots
 *            are counted from the element before its first one, which is dropped; plan[4] to plan[6] and
 *            the choice of substituted slots are those of rows of cols + 1 elements, plan[5], plan[6]
 *            count the steps that are whole for a row read either way
 */
int mfr_rows_plan(size_t x_addr, int dtype, size_t rows, size_t cols, size_t row_stride, int cus,
                  unsigned long long plan[12]);

/*
 * Geometry of the per-row kernels for mfr_sum_rows_ex(x, dtype, rows, cols,
 * row_stride, out, t, stream) on a device with `cus` compute units (pure host
 * arithmetic, no device access): every row is reduced as a single array is
 * (Section 5.2), plan[1] blocks sharing a row.  Returns 1 and fills plan[], 0
 * if t == NULL and the many-rows kernel takes the call (see mfr_rows_plan),
 * negative status on invalid arguments (rows == 0 and cols == 0 included).
 *   plan[0]  threads per block          plan[1]  blocks per row
 *   plan[2]  chain_R                    plan[3]  chains in flight per wave
 *   plan[4]  full chains per row (of a row that starts on a 16-byte boundary when plan[7] is 1)
 *   plan[5]  stagger: row r reads its chains starting r * plan[5] bytes further on, rounded to whole chains
 *            and taken modulo the row's chains, and wraps round (0: every row from its first chain)
 *   plan[6]  bytes of LDS that the launch asks for without using them, which limits the blocks resident
 *            per compute unit (0: no limit)
 *   plan[7]  1 if the rows differ in 16-byte phase and each block works out the slots of its own row
 */
int mfr_rows_geometry(size_t x_addr, int dtype, size_t rows, size_t cols, size_t row_stride, const mfr_tuning *t,
                      int cus, unsigned long long plan[8]);

/*
 * Frees the scratch that calls on `stream` of the current device have left
 * with the library (block partials, combine slots, the recurrence variant's
 * level buffers), after synchronising the stream.  For streams that are about
 * to be destroyed, or to hand the memory back; a later call on the stream
 * allocates again.  Returns MFR_OK also when the stream holds none.  Must not
 * overlap with other libmfreduce calls on the same stream, and not be called
 * while the stream is being captured into a graph.
 */
int mfr_release_scratch(hipStream_t stream);

/* Static text for a status code. */
const char *mfr_strerror(int status);

/* Text of the most recent HIP error seen by the calling thread ("" if none). */
const char *mfr_last_hip_error(void);

/* major * 10000 + minor * 100 + patch */
int mfr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MFREDUCE_H */
