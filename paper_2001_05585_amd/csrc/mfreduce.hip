// libmfreduce host side: argument checks, geometry, scratch, launches, C ABI.
// The kernels are in mfr_kernels.hpp, instantiated per element type in
// launch_f16.hip / launch_bf16.hip / launch_f32.hip.

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

#include "mfr_kernels.hpp"

namespace {

using mfr::Plan;
using mfr::SumArgs;
using mfr::uint4v;

// Second launch of the two-launch combine: block r adds the partials of row r.
__global__ void __launch_bounds__(1024) combine_kernel(const float *partials, unsigned int count, float *out)
{
    __shared__ double wave_partials_f64[mfr::kMaxWavesPerBlock];
    const double total = mfr::block_sum_f64(partials + (size_t)blockIdx.x * count, count, wave_partials_f64);
    if (threadIdx.x == 0) out[blockIdx.x] = (float)total;
}

__global__ void store_zero_kernel(float *out, unsigned long long count)
{
    const unsigned long long step = (unsigned long long)gridDim.x * blockDim.x;
    for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += step) out[i] = 0.f;
}

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
    size_t partials_capacity = 0;   // floats
    unsigned int *slots = nullptr;      // single-launch combine: one word per block, all zero between calls
    size_t slots_capacity = 0;
    unsigned short *levels = nullptr;   // recurrence variant: the binary16 partials of two levels
    size_t levels_capacity = 0;
    // Buffers that a larger one has replaced.  A call copies the current pointers under the mutex
    // and launches after dropping it, and work already enqueued (or captured into a graph) keeps
    // the addresses it was given, so a replaced buffer is kept until mfr_release_scratch.
    std::vector<void *> retired;
    // Held by a call from before it reads the pointers above until its last launch is enqueued: the
    // launches of one call (sum kernel + combine kernel, the levels of the recurrence) then sit next
    // to each other in the stream even when several host threads enqueue on it, so no other call's
    // kernel can overwrite the scratch between them.
    std::mutex launch_mutex;
};

std::mutex g_mutex;
DeviceInfo g_devices[64];
std::map<std::pair<int, hipStream_t>, Scratch> g_scratch;

constexpr int kDefaultBlock = 256;
// Six KiB of loads in flight per wave (two chains of three tiles), one wave per SIMD, is where the
// chip streams fastest: 75.7 us for 512 MiB against 77.2 us with eight KiB and 89 us with four.
constexpr int kDefaultR = 3;
constexpr int kDefaultR_shfl = 6;              // the conventional kernel: one group of six loads
constexpr int kDefaultR_f32 = 7;               // binary32: one chain of seven tiles (75.9 us; two chains of three: 80 us)
// A single array of more than 96 KiB and at most 256 MiB, all of block size, chain length and chains
// in flight left to the library: 128-thread blocks and one chain of eight tiles, i.e. 8 KiB contiguous
// per wave and step.  Such calls spend a large part of their time getting started and finishing, and
// this geometry shortens both (64 MiB: 21.3 us against 22.0; 32 MiB: 7.8 against 8.3; 8 MiB: 4.5
// against 4.8); from 512 MiB on six KiB per wave in two chains streams faster (75.6 us against 76.5).
constexpr unsigned long long kMidSizeMinBytes = 96ull << 10;
constexpr unsigned long long kMidSizeMaxBytes = 256ull << 20;
constexpr int kMidSizeBlock = 128;
constexpr int kMidSizeR = 8;
constexpr int kDefaultWavesPerCU = 4;          // one wave per SIMD
constexpr long long kSingleLaunchAutoMax = 2048;   // AUTO: larger grids combine with a second launch
constexpr long long kSingleLaunchHardMax = 65536;  // single-launch combine is not offered beyond this
constexpr size_t kMaxRowsPerLaunch = 65535;    // gridDim.y limit
constexpr unsigned long long kRowsApartBytes = 1ull << 20;    // few long rows are read at addresses this far apart (or a multiple)
constexpr unsigned long long kOneBlockMaxChains = 32;   // library defaults: arrays this short get one block
// Inputs that fit in the eight 4 MiB L2s may be resident there (a reduction often follows the kernel
// that produced its input): they are read with ordinary loads, which hit in L2 (20 % faster at 32 MiB
// when resident, 3-6 % slower when not).  Larger inputs stream through with non-temporal loads (8 %
// faster from HBM).
constexpr size_t kTemporalBytes = (size_t)32 << 20;

// The default block size and chain length, after the optional environment override (MFR_BLOCK,
// MFR_R; read once per process).  `valid` is false if a variable is set to something unusable:
// every call that relies on the default then fails, rather than silently running another geometry.
struct DefaultGeometry {
    int block;
    int chain_R;      // 0: the per-type default
    bool valid;
    bool overridden;  // a variable is set: the library's own choices of block size stand back
};

const DefaultGeometry &default_geometry()
{
    static const DefaultGeometry g = [] {
        DefaultGeometry d = {kDefaultBlock, 0, true, getenv("MFR_BLOCK") != nullptr || getenv("MFR_R") != nullptr};
        if (const char *e = getenv("MFR_BLOCK")) {
            char *end = nullptr;
            const long v = strtol(e, &end, 10);
            if (end == e || *end != '\0' || !(v == 32 || v == 64 || v == 128 || v == 256 || v == 512 || v == 1024)) d.valid = false;
            else d.block = (int)v;
        }
        if (const char *e = getenv("MFR_R")) {
            char *end = nullptr;
            const long v = strtol(e, &end, 10);
            if (end == e || *end != '\0' || v < 1 || v > 8) d.valid = false;
            else d.chain_R = (int)v;
        }
        return d;
    }();
    return g;
}

void resolve_load_policy(mfr_tuning *t, size_t bytes)
{
    if (t->nontemporal == 0) t->nontemporal = bytes <= kTemporalBytes ? 1 : 2;
}
// The tiled rows kernel takes over from this many rows on; long rows (one row per tile) from fewer.
constexpr size_t kRowsTiledMinRows = 1024;
constexpr size_t kRowsTiledMinLongRows = 512;
// Rows of this many bytes or more are walked one per wave, 4 KiB per step, instead of four side by
// side, 1 KiB each per step: with a power-of-two row stride the four pieces of a step would fall
// into the same memory channels.
constexpr size_t kRowsTiledLongRowBytes = 4096;
constexpr size_t kRowsTiledMaxRowBytes = 16384;

// Chains in flight that bring R * U closest to 6 tiles (6 KiB of loads per wave,
// the measured optimum), the larger count on a tie.
int default_in_flight(int R)
{
    static const int kByR[9] = {0, 6, 3, 2, 2, 1, 1, 1, 1};
    return kByR[R < 1 ? 1 : (R > 8 ? 8 : R)];
}

bool valid_block(int b)
{
    return b == 32 || b == 64 || b == 128 || b == 256 || b == 512 || b == 1024;
}

unsigned elem_size(int dtype) { return dtype == MFR_DTYPE_F32 ? 4u : 2u; }

bool valid_dtype(int dtype)
{
    return dtype == MFR_DTYPE_F16 || dtype == MFR_DTYPE_BF16 || dtype == MFR_DTYPE_F32;
}

// Fills in defaults and checks ranges; no HIP calls.  `single_array_bytes`: size of the input when
// the call sums one array (selects the size-dependent defaults), 0 otherwise.
int resolve_tuning(const mfr_tuning *in, int dtype, mfr_tuning *t, unsigned long long single_array_bytes = 0)
{
    mfr_tuning z;
    memset(&z, 0, sizeof z);
    if (in) z = *in;
    if (!valid_dtype(dtype)) return MFR_ERR_INVALID_ARG;
    if (z.block_threads == 0 || z.chain_R == 0) {
        const DefaultGeometry &g = default_geometry();
        if (!g.valid) return MFR_ERR_INVALID_ARG;
        if (z.block_threads == 0 && z.chain_R == 0 && z.chains_in_flight == 0 && !g.overridden &&
            z.kernel != MFR_KERNEL_SPLIT && single_array_bytes > kMidSizeMinBytes && single_array_bytes <= kMidSizeMaxBytes) {
            z.block_threads = kMidSizeBlock;
            z.chain_R = kMidSizeR;
            z.chains_in_flight = 1;
        }
        if (z.block_threads == 0) z.block_threads = g.block;
        if (z.chain_R == 0)
            z.chain_R = g.chain_R ? g.chain_R
                        : (z.kernel == MFR_KERNEL_SHFL ? kDefaultR_shfl : (dtype == MFR_DTYPE_F32 ? kDefaultR_f32 : kDefaultR));
    }
    if (!valid_block(z.block_threads)) return MFR_ERR_INVALID_ARG;
    if (z.block_threads == 32 && dtype != MFR_DTYPE_F16) return MFR_ERR_INVALID_ARG;
    if (z.chain_R < 1 || z.chain_R > 8) return MFR_ERR_INVALID_ARG;
    if (z.grid_blocks < MFR_GRID_ONE_CHAIN) return MFR_ERR_INVALID_ARG;
    if (z.kernel != MFR_KERNEL_MFMA && z.kernel != MFR_KERNEL_SHFL && z.kernel != MFR_KERNEL_SPLIT)
        return MFR_ERR_INVALID_ARG;
    if (z.kernel == MFR_KERNEL_SPLIT && (dtype != MFR_DTYPE_F16 || z.block_threads == 32)) return MFR_ERR_INVALID_ARG;
    if (z.split_permille < 0 || z.split_permille > 1000) return MFR_ERR_INVALID_ARG;
    if (z.kernel != MFR_KERNEL_SPLIT && z.split_permille != 0) return MFR_ERR_INVALID_ARG;
    if (z.chains_in_flight == 0) z.chains_in_flight = default_in_flight(z.chain_R);
    const int u = z.chains_in_flight;
    if (!(u == 1 || u == 2 || u == 3 || u == 4 || u == 6 || u == 8)) return MFR_ERR_INVALID_ARG;
    if (u * z.chain_R > 16) return MFR_ERR_INVALID_ARG;
    if (z.nontemporal < 0 || z.nontemporal > 2) return MFR_ERR_INVALID_ARG;   // 0 is resolved per call size
    if (z.combine < 0 || z.combine > 2) return MFR_ERR_INVALID_ARG;
    *t = z;
    return MFR_OK;
}

// Slot / chain arithmetic for n elements of `esize` bytes starting at byte address x_addr.
void plan_region(size_t n, size_t x_addr, unsigned esize, const mfr_tuning &t, Plan *p)
{
    memset(p, 0, sizeof *p);
    p->half = t.block_threads == 32;
    p->threads = p->half ? 64 : t.block_threads;
    p->waves = p->threads / 64;
    const unsigned int ts = p->half ? 32u : 64u;
    mfr::region_fields(n, (unsigned int)((x_addr & 15u) / esize), 16u / esize, ts * (unsigned)t.chain_R, &p->a);
    p->chains = p->a.chains;
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

// Library defaults, single array of at most kOneBlockMaxChains chains: one block with a wave per
// chain (up to 16 waves).  Rewrites the block size and the grid of *t and returns true if so.
bool one_block_default(unsigned long long chains, mfr_tuning *t)
{
    if (default_geometry().overridden || chains > kOneBlockMaxChains) return false;
    int waves = 1;
    while ((unsigned long long)waves < chains && waves < 16) waves *= 2;
    t->block_threads = 64 * waves;
    t->grid_blocks = 1;
    return true;
}

// Blocks per row.  `rows` rows share the persistent grid.
long long grid_blocks_for(const Plan &p, const mfr_tuning &t, int cus, size_t rows)
{
    const unsigned long long need = (p.chains + (unsigned)p.waves - 1ull) / (unsigned)p.waves;
    unsigned long long g;
    if (t.grid_blocks == MFR_GRID_ONE_CHAIN) {
        g = need;
    } else if (t.grid_blocks == MFR_GRID_AUTO) {
        int per_cu = kDefaultWavesPerCU / p.waves;
        if (per_cu < 1) per_cu = 1;
        g = (unsigned long long)cus * (unsigned)per_cu;
        if (rows > 1) g = g / rows;              // rounded down: a second round of blocks costs more than idle CUs
        if (g > need) g = need;
    } else {
        g = (unsigned long long)t.grid_blocks;
    }
    if (g < 1ull) g = 1ull;
    if (g > 0x7fffffffull) return -1;
    return (long long)g;
}

// One to two rows per SIMD (binary32: up to 1.6), rows of 64 KiB and more: a one-wave block per row, all resident at
// once, each with as many tiles in flight as bring the device to about one wave of 6 KiB per SIMD, instead of
// 256-thread blocks in rounds.  512 MiB of binary16 rows: 1030 rows 75 -> 82 % of 8 TB/s, 1100 rows 79 -> 85 %, 1400
// rows 78 -> 85 %, 1800 rows 80 -> 86 %, +3.5 points on average over 1024 to 2047 rows; binary32 +3 up to 1600 rows
// and -0.4 from there on (left as it was); 1500 rows of 80 KB 73 -> 81 %.  Shorter rows (16 and 32 KiB) gain
// nothing on average.
bool one_wave_per_row(size_t rows, size_t row_bytes, unsigned esize, int cus)
{
    const size_t simds = (size_t)cus * 4u;
    return rows >= simds && rows < (esize == 4 ? simds + simds * 5u / 8u : simds * 2u) && row_bytes >= 65536u;
}

// Block size for `rows` rows of row_bytes bytes sharing the persistent grid (one wave per SIMD in
// all): the CUs hold cus * 256 / block blocks; a row gets floor(that / rows) of them (at least one).
// Fewest rounds of blocks first, then the fullest round; a smaller block must fill more than a
// tenth better to win.  With more rows than the CUs hold 64-thread blocks every row is one block
// anyway and the row's length decides (measured with 512 MiB of rows of 4 KiB to 512 KiB).
int block_threads_for_rows(size_t rows, size_t row_bytes, unsigned esize, int cus)
{
    if (one_wave_per_row(rows, row_bytes, esize, cus)) return 64;
    if (rows >= (size_t)cus * 4u) return row_bytes < 12288u ? 64 : (row_bytes < 32768u ? 128 : 256);
    int best_block = 256;
    unsigned long long best_rounds = 0;
    double best_fill = 0.0;
    for (int block = 256; block >= 64; block /= 2) {
        const unsigned long long slots = (unsigned long long)cus * (256u / (unsigned)block);
        unsigned long long g = slots / rows;
        if (g < 1) g = 1;
        const unsigned long long blocks = g * rows;
        const unsigned long long rounds = (blocks + slots - 1) / slots;
        const double fill = (double)blocks / (double)(rounds * slots);
        if (block == 256 || rounds < best_rounds || (rounds == best_rounds && fill > best_fill + 0.1)) {
            best_block = block;
            best_rounds = rounds;
            best_fill = fill;
        }
    }
    return best_block;
}

// Many rows of 12 KiB and more through the per-row kernels (library defaults): the hardware would keep as many
// blocks resident per CU as registers allow, 8 waves per SIMD, and that many streams at once slow each other
// down.  The launch asks for enough LDS per block that only 8 waves per CU fit (rows of 64 KiB and more: two
// 256-thread blocks), 12 (shorter rows of a 16-bit type: six 128-thread or three 256-thread blocks) or 16
// (shorter binary32 rows, whose waves have one chain in flight); the LDS is not used.  binary16: 16 KiB rows
// 86 -> 90 % of 8 TB/s, 32 KiB rows 85 -> 89 %, 64 KiB rows 84 -> 88 %, 128 KiB rows 84 -> 86 %; binary32: 16 and
// 32 KiB rows 86 / 87 -> 88 / 89 %, 64 KiB rows 85 -> 87 %.  Only for rows made of whole 16-byte slots:
// a row with a head slot pays a round trip of element-wise loads, which fewer resident blocks hide worse (32 KiB
// rows one element off a boundary: 86 % unlimited, 68 % with 12 waves), and so does a row with a ragged last slot
// (-6 points).  Shorter rows (64-thread blocks) do best unlimited.  Returns 0 (no limit) also when the launch has
// fewer blocks than two rounds of that many, or when its last round would be so empty that over 4 % of the time
// went into it (1061 rows of 500 KB: two rounds of 512 blocks and one of 37).
unsigned int resident_limit_lds(size_t rows, unsigned long long blocks_per_row, size_t row_bytes, unsigned esize,
                                bool whole_slots, int waves_per_block, int cus)
{
    if (rows < 2 || waves_per_block < 1 || row_bytes < 12288u || !whole_slots) return 0;
    const unsigned waves_per_cu = row_bytes >= 65536u ? 8u : (esize == 2u ? 12u : 16u);
    unsigned long long per_cu = waves_per_cu / (unsigned)waves_per_block;
    if (per_cu < 1) per_cu = 1;
    const unsigned long long blocks = (unsigned long long)rows * blocks_per_row, round = per_cu * (unsigned)cus;
    if (blocks < 2ull * round) return 0;
    const unsigned long long rounds = (blocks + round - 1ull) / round;
    if (blocks * 100ull < rounds * round * 96ull) return 0;
    const unsigned long long lds_per_cu = 160ull * 1024ull;
    unsigned long long want = lds_per_cu / per_cu - 1536ull;      // per_cu blocks fit, per_cu + 1 do not
    if (want > 61440ull) want = 61440ull;                         // what a launch may ask for without more ado
    return (unsigned int)(want / 256ull * 256ull);
}

// Capacity doubles until it covers `need`.  The buffer that is outgrown is not freed here (see
// Scratch::retired): all retired buffers of a stream together are smaller than its current one.
int grow(void **mem, size_t *capacity, size_t need, size_t elem, size_t floor_count, bool zero,
         std::vector<void *> *retired)
{
    if (*capacity >= need) return MFR_OK;
    size_t cap = *capacity ? *capacity : floor_count;
    while (cap < need) cap *= 2;
    void *fresh = nullptr;
    MFR_HIP(hipMalloc(&fresh, cap * elem));
    if (zero) {
        const hipError_t e = hipMemset(fresh, 0, cap * elem);
        if (e != hipSuccess) { (void)hipFree(fresh); return hip_fail(e, "hipMemset(scratch)"); }
        // the fill runs on the null stream; the caller's stream need not wait for that stream by itself
        const hipError_t e2 = hipStreamSynchronize(nullptr);
        if (e2 != hipSuccess) { (void)hipFree(fresh); return hip_fail(e2, "hipStreamSynchronize(scratch fill)"); }
    }
    if (*mem) retired->push_back(*mem);
    *mem = fresh;
    *capacity = cap;
    return MFR_OK;
}

// Where a call's block partials (two-launch combine) and slots (single-launch combine) live: the stream's library-owned buffers
// (allocated or enlarged here if need be), or a fixed region that the caller of sum_rows_impl
// hands in and that is never enlarged.
struct ScratchView {
    float *partials = nullptr;
    size_t partials_capacity = 0;
    unsigned int *slots = nullptr;
    size_t slots_capacity = 0;
    std::mutex *launch_mutex = nullptr;     // fixed regions: the mutex that keeps one call's launches together
};

// Locks the stream's launch mutex into *launch_lock (the caller keeps it until its last launch).
int get_scratch(int dev, hipStream_t stream, size_t partials, size_t slots, ScratchView *out,
                std::unique_lock<std::mutex> *launch_lock)
{
    Scratch *entry = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        entry = &g_scratch[std::make_pair(dev, stream)];      // map nodes do not move
    }
    *launch_lock = std::unique_lock<std::mutex>(entry->launch_mutex);
    std::lock_guard<std::mutex> lock(g_mutex);
    Scratch &s = *entry;
    int st = grow((void **)&s.partials, &s.partials_capacity, partials, sizeof(float), 4096, false, &s.retired);
    if (st != MFR_OK) return st;
    st = grow((void **)&s.slots, &s.slots_capacity, slots, sizeof(unsigned int), 1024, true, &s.retired);
    if (st != MFR_OK) return st;
    out->partials = s.partials;
    out->partials_capacity = s.partials_capacity;
    out->slots = s.slots;
    out->slots_capacity = s.slots_capacity;
    return MFR_OK;
}

hipError_t launch_dtype(int dtype, const Plan &p, dim3 grid, const mfr_tuning &t, hipStream_t stream)
{
    switch (dtype) {
    case MFR_DTYPE_F16: return mfr::launch_sum_f16(p, grid, t, stream);
    case MFR_DTYPE_BF16: return mfr::launch_sum_bf16(p, grid, t, stream);
    case MFR_DTYPE_F32: return mfr::launch_sum_f32(p, grid, t, stream);
    default: return hipErrorInvalidValue;
    }
}

// The array's span (rows - 1) * row_stride + cols must stay below 2^60 elements, so that byte
// offsets cannot wrap.
bool span_fits(size_t rows, size_t cols, size_t row_stride)
{
    const unsigned long long limit = 1ull << 60;
    if (cols > limit) return false;
    if (rows <= 1) return true;
    return row_stride <= (limit - cols) / (rows - 1);
}

// Shape of the tiled rows kernel for rows x cols elements of `esize` bytes at byte address x_addr,
// rows row_stride elements apart.  Returns false when the per-row kernels are the better choice:
// few rows (they cannot fill the device here, a grid per row can) or very long ones.
bool plan_rows_tiled(size_t x_addr, unsigned esize, size_t rows, size_t cols, size_t row_stride, int cus,
                     mfr::RowsTiledShape *s, unsigned *grid)
{
    if (rows < 2 || cols == 0) return false;
    const unsigned long long per_slot = 16u / esize;
    const unsigned long long stride_bytes = (unsigned long long)row_stride * esize;
    const unsigned long long row_bytes = (unsigned long long)cols * esize;
    // rows this long are streamed as well or better by a grid of blocks per row
    if (row_bytes >= kRowsTiledMaxRowBytes) return false;
    // 128-bit loads at 2-byte alignment lose a quarter of the rate or more.  When some rows of a 16-bit type
    // start at such addresses, those rows are read from one element earlier, and every row is planned as one
    // element longer (no row then consists of whole steps): 512-byte rows 2 bytes off a boundary 67 -> 82 %,
    // 1000-byte ones 64 -> 83 %, 200-byte ones 53 -> 77 %, rows of 257 elements 75 -> 78 %.  From 4 KiB rows on
    // the per-row kernels, which read aligned slots whatever the rows' phases, do as well (6000-byte rows 78 %
    // against 81 %, 8192-byte rows 79 % against 78 %).
    const bool shift = esize == 2u && ((x_addr & 2u) != 0u || (stride_bytes & 2u) != 0u);
    if (shift && row_bytes >= kRowsTiledLongRowBytes) return false;
    const unsigned long long held_bytes = row_bytes + (shift ? 2ull : 0ull);      // what a row's steps have to hold
    int lp = 0;
    while (lp < 4 && (64ull << lp) < held_bytes) ++lp;
    int d = 1, gf = 8;
    // Rows of up to four whole 1 KiB steps (P = 16), or one 512-byte step (P = 8), and at most 256 bytes more:
    // plain steps, and the rests of all rows of an iteration in tail tiles (P_t = 1, 2 or 4 columns per row for
    // rests of up to 64, 128, 256 bytes) instead of a masked step of their own (520-byte rows 83 % against 69 %,
    // 1040-byte rows 88 % against 74 %, 1200-byte rows 87 % against 76 %, 2060-byte rows 85 % against 76 %,
    // 2300-byte rows 87 % against 78 %, 4200-byte rows 85 % against 81 %).  One plain step: eight groups side by
    // side; several: four (as for unmasked rows of these steps), with the steps written out so that the tail
    // tiles are loaded once per iteration.  Rows that are whole steps of a narrower shape keep that shape; several
    // 512-byte steps gain nothing.  Shifted rows of 256 to 318 bytes take one 256-byte step (P = 4) and a tail
    // tile (256-byte rows 2 bytes off a boundary 67 -> 79 %).
    int tail_lp = 0, tail_lpt = 0;
    if (row_bytes < 5120ull && (shift || row_bytes % 256ull != 0)) {
        auto rest_after = [&](unsigned long long step) { return held_bytes - row_bytes / step * step; };
        unsigned long long rest = 0;
        if (row_bytes >= 1024ull) {
            rest = rest_after(1024ull);
            if (rest > 0 && rest <= 256ull) tail_lp = 4;
        } else if (row_bytes >= 512ull) {
            rest = rest_after(512ull);
            if (rest > 0 && rest <= 256ull) tail_lp = 3;
        } else if (shift && row_bytes >= 256ull) {
            rest = rest_after(256ull);
            if (rest <= 64ull) tail_lp = 2;
        }
        tail_lpt = rest <= 64ull ? 0 : (rest <= 128ull ? 1 : 2);
    }
    bool tail = false;
    if (tail_lp != 0 && rows >= kRowsTiledMinRows) {
        lp = tail_lp;
        tail = true;
        gf = (tail_lp == 2 || row_bytes >= 2048ull) ? 4 : 8;
    } else if (rows >= kRowsTiledMinRows && row_bytes < kRowsTiledLongRowBytes) {
        // Rows over 512 bytes: a step of P = 16 is 1 KiB, and a row that ends early in its last step
        // leaves the rest of that step's loads empty.  Rows that are whole steps of a narrower shape
        // take that shape, unmasked (768-byte rows 89 % against 69 %).
        const unsigned long long covered = (held_bytes + 1023ull) / 1024ull * 1024ull;      // in 1 KiB steps
        if (held_bytes > 512 && held_bytes % 1024ull != 0) {
            if (held_bytes % 512ull == 0) lp = 3;
            else if (held_bytes % 256ull == 0) lp = 2;
        }
        // Two steps are in flight per wave: 8 KiB with four groups, 16 KiB with eight.  Unmasked rows
        // made of 256- or 512-byte steps do better with four (256-element fp16 rows 88 % against 84 %);
        // shorter rows and masked rows (100-element rows 67 % against 78 %) with eight.
        const bool whole_steps = !shift && row_bytes % (64ull << lp) == 0;
        if (lp == 4 || (lp >= 2 && whole_steps)) gf = 4;
        // A masked last step of P = 16 carries fewer bytes than it has loads: when it is the only step,
        // or when the row fills under 80 % of its steps, eight groups keep enough of them in flight
        // (800-byte rows 87 % against 70 %, 2200-byte rows 78 % against 72 %).
        if (lp == 4 && !whole_steps && (covered == 1024ull || held_bytes * 100ull < covered * 80ull)) gf = 8;
    } else if (lp == 4 && rows >= kRowsTiledMinLongRows) {
        d = 4; gf = 1;
        if (shift) { d = 1; gf = 4; }            // shifted rows: one tile per step
        // A step of four tiles leaves up to 4 KiB of its last step empty.  Rows that would waste
        // more than a fifth of their steps go four side by side, 1 KiB each per step, unless their
        // stride is a multiple of 1 KiB (the four pieces would share memory channels).
        const unsigned long long steps4 = (row_bytes + 4095ull) / 4096ull;
        if (row_bytes * 5ull < steps4 * 4096ull * 4ull && (stride_bytes % 1024ull) != 0) { d = 1; gf = 4; }
    } else {
        return false;
    }
    const unsigned long long p = 1ull << lp;
    const unsigned long long rows_per_iter = (unsigned long long)gf * (16ull / p);
    const unsigned long long slots_per_step = 4ull * p * (unsigned)d;
    const unsigned long long slots = (cols + (shift ? 1ull : 0ull) + per_slot - 1ull) / per_slot;
    const unsigned long long plain_hi = (cols / per_slot) / slots_per_step;       // >= batches - 1
    const unsigned long long batches = tail ? plain_hi : (slots + slots_per_step - 1ull) / slots_per_step;
    if (batches > 0xffffffffull) return false;
    s->log2_p = lp;
    s->tiles_per_step = d;
    s->groups = gf;
    s->iters = (rows + rows_per_iter - 1ull) / rows_per_iter;
    s->batches = (unsigned int)batches;
    s->plain_hi = (unsigned int)plain_hi;
    s->all_plain = plain_hi == batches;
    s->tail = tail;
    s->tail_log2_p = tail ? tail_lpt : 0;
    s->shift = shift;
    // Rows whose last slot would end past the array's span are not for this kernel: row r reads
    // bytes [r * stride, r * stride + 16 * slots) from x (a shifted row 2 bytes less at either end), the span
    // ends at (rows - 1) * stride + row_bytes.
    const unsigned long long span = (rows - 1ull) * stride_bytes + row_bytes;
    unsigned long long tail_rows = 0;
    while (tail_rows < rows && (rows - 1ull - tail_rows) * stride_bytes + 16ull * slots > span) ++tail_rows;
    if (tail_rows >= rows) return false;
    s->row_hi = rows - tail_rows;
    // 256-thread blocks: one wave per SIMD
    unsigned long long g = (unsigned long long)cus;
    // A single masked step that is under 69 % full, and 256-byte steps with a tail tile: two blocks per CU, so
    // that more loads are in flight while so many of them carry nothing (32-byte rows 66 -> 77 %, binary32 rows
    // of 160 bytes 72 -> 77 %, of 320 bytes 77 -> 80 %); everywhere else a second block costs 3 to 6 points.
    const unsigned long long step_bytes = 64ull * p * (unsigned)d;
    if ((batches == 1ull && plain_hi == 0ull && held_bytes * 100ull < step_bytes * 69ull) || (tail && lp == 2)) g *= 2ull;
    if (g * 4ull > s->iters) g = (s->iters + 3ull) / 4ull;
    *grid = (unsigned)g;
    return true;
}

int fill_zero(float *out, size_t count, hipStream_t stream)
{
    const size_t want = (count + 255) / 256;
    const unsigned blocks = (unsigned)(want < 65536 ? want : 65536);      // the kernel strides over the rest
    hipLaunchKernelGGL(store_zero_kernel, dim3(blocks), dim3(256), 0, stream, out, (unsigned long long)count);
    MFR_HIP(hipGetLastError());
    return MFR_OK;
}

// Geometry of the per-row kernels for a batched call (pure host arithmetic): block size, blocks per row, chain
// shape, LDS that limits residency, stagger.  `t` comes in resolved and goes out as launched; `defaults` says that
// the caller left the tuning to the library.
int per_row_geometry(size_t x_addr, unsigned esize, size_t rows, size_t cols, size_t row_stride, bool defaults, int cus,
                     mfr_tuning *t_io, Plan *p_out, long long *grid_out)
{
    mfr_tuning &t = *t_io;
    Plan &p = *p_out;
    // rows that all have the same 16-byte phase can be read in aligned slots
    const bool same_phase = rows == 1 || ((row_stride * esize) & 15u) == 0;
    // Row counts that do not divide the CUs well: smaller blocks, more of them per CU, fill the
    // device in one round (300 rows: 86 % with 64-thread blocks against 70 % with 256-thread ones).
    if (defaults && rows > 1) {
        t.block_threads = block_threads_for_rows(rows, cols * esize, esize, cus);
        // Row counts that leave SIMDs without a wave (a few hundred rows): the waves there are keep more loads in
        // flight each, so that the device as a whole has about what one wave of 6 KiB per SIMD would have
        // (520 rows of 1 MiB: 57 -> 78 % of 8 TB/s, 600 rows 64 -> 82 %, 700 rows 70 -> 81 %, 260 rows 75 -> 83 %).
        // 8 KiB per wave already when 6 KiB would leave the device under 92 % of that (300 rows of 1.7 MiB 80 -> 86 %,
        // 450 rows 81 -> 85 %, 900 rows 81 -> 84 %; 1000 rows, at 98 %, are better off with 6 KiB: 84 against 81.5 %),
        // as one chain for binary32 (2 points better on average) and as two for the 16-bit types.
        // A few rows more than half the SIMDs: two one-wave blocks per row with 6 KiB each instead of one with 12 KiB.
        // binary32, 513 to 640 rows: 516 to 540 rows of 1 MiB 70 -> 82 %, 600 rows 77.5 -> 82.5 %, 640 rows 80 -> 83 %
        // (two of 28 row lengths measured lose 6 to 9 points).  16-bit types, 513 to 544 rows: 520 rows of 1 MiB
        // 76 -> 80 %, +1.2 points on average; from there on no gain on average and single lengths 14 points lower.
        if (!default_geometry().overridden && t.kernel == MFR_KERNEL_MFMA) {
            const unsigned long long slots = (unsigned long long)cus * (256u / (unsigned)t.block_threads);
            unsigned long long per_row = slots / rows;
            if (per_row < 1) per_row = 1;
            if (per_row == 1 && t.block_threads == 64 && 2ull * rows <= slots + slots / (esize == 4 ? 4ull : 16ull) &&
                cols * esize >= 65536u) {
                per_row = 2;
                t.grid_blocks = 2;
                t.chain_R = 6;              // as one chain: +0.5 points on average against two chains of three tiles, and
                t.chains_in_flight = 1;     // the unluckiest row lengths reach 68-77 % instead of 62-75 %
            }
            const unsigned long long waves = rows * per_row * ((unsigned)t.block_threads / 64u);
            const unsigned long long want = 6ull * 4ull * (unsigned)cus;      // tiles in flight on the device
            if (want > 12ull * waves) { t.chain_R = 8; t.chains_in_flight = 2; }
            else if (want > 8ull * waves) { t.chain_R = 6; t.chains_in_flight = 2; }
            else if (2ull * want > 13ull * waves) {
                if (esize == 4) { t.chain_R = 8; t.chains_in_flight = 1; }
                else { t.chain_R = 4; t.chains_in_flight = 2; }
            }
            else if (one_wave_per_row(rows, cols * esize, esize, cus)) {
                // more waves than SIMDs: 3 KiB each from 1.66 waves per SIMD on, 4 KiB from 1.2 on (6 KiB below that)
                if (37ull * waves > 10ull * want) { t.chain_R = 3; t.chains_in_flight = 1; }
                else if (5ull * waves > want) { t.chain_R = 4; t.chains_in_flight = 1; }
            }
        }
    }
    const size_t batch = rows < kMaxRowsPerLaunch ? rows : kMaxRowsPerLaunch;

    // Rows are addressed in aligned slots counted from the boundary at or below their first element
    // (the head slot is read element-wise).  Rows that share their 16-byte phase share the slot
    // arithmetic done here; rows of differing phase are planned as if they started on a boundary
    // (which gives the largest number of chains), and each block redoes the arithmetic for its row.
    plan_region(cols, same_phase ? x_addr : 0, esize, t, &p);
    // A short single array is summed by one block with a wave per chain (up to 16 waves, two chains
    // each): combining several blocks costs three dependent device-scope round trips, 1.6 us, which a
    // call replayed from a graph would see in full (1.9 us against 3.4 us per call).
    if (defaults && rows == 1 && cols * esize <= kMidSizeMinBytes && one_block_default(p.chains, &t))
        plan_region(cols, x_addr, esize, t, &p);
    p.a.per_row_phase = same_phase ? 0u : 1u;
    const long long grid = grid_blocks_for(p, t, cus, batch);
    if (grid < 1) return MFR_ERR_INVALID_ARG;
    *grid_out = grid;
    p.dynamic_lds = resident_limit_lds(defaults ? rows : 0, (unsigned long long)grid, cols * esize, esize,
                                       same_phase && (x_addr & 15u) == 0 && ((cols * esize) & 15u) == 0, p.waves, cus);
    // Library defaults, several rows: row r starts r * rotate_bytes further on, rounded to whole chains (and
    // wraps round), with rotate_bytes what the row pitch lacks to the next multiple of 1 MiB: the addresses the
    // rows are read at, at any one time, then lie a multiple of 1 MiB apart whatever the row pitch is (to within
    // a chain).  The memory channels take such a pattern evenly; with the rows all read at the same distance
    // from their starts, some pitches put them onto the same channels (145 rows of 3 702 544 bytes: 63 -> 83 % of
    // 8 TB/s, 143 rows of 3 754 336 bytes 60 -> 83 %, 339 rows 74 -> 83 %; mean over 95 random shapes of 2 to 1023
    // rows 82.6 -> 83.9 %).  Granularities of 512 KiB to 4 MiB do the same, 64 KiB less (83.3 %); four evenly spaced
    // starting points gave 83.0 %, a pseudo-random start per row costs rows whose pitch was fine up to 14 points.
    // One to two rows per SIMD with a one-wave block each: same mean with and without (84 shapes), but the
    // unluckiest are lifted (1024 rows of 520 288 bytes 65 -> 82 %, of 130 072 floats 65 -> 86 %; 24 -> 19 shapes
    // under 78 %).  More rows run in rounds, not side by side, and are left alone.
    p.a.rotate_bytes = 0ull;
    if (defaults && rows > 1 && p.a.chains > 16ull &&
        (rows < (size_t)cus * 4u || one_wave_per_row(rows, cols * esize, esize, cus))) {
        const unsigned long long pitch = (unsigned long long)row_stride * esize;
        p.a.rotate_bytes = (pitch + kRowsApartBytes - 1ull) / kRowsApartBytes * kRowsApartBytes - pitch;
    }
    return MFR_OK;
}

// rows sums of cols elements each; consecutive rows are row_stride elements apart.
// `fixed`: if not null, the block partials and slots live there and nothing is allocated; a call
// that needs more than it holds fails with MFR_ERR_SCRATCH_LIMIT.
int sum_rows_impl(const void *x, int dtype, size_t rows, size_t cols, size_t row_stride, float *out,
                  const mfr_tuning *tin, hipStream_t stream, const ScratchView *fixed = nullptr,
                  unsigned long long *stamps = nullptr, size_t stamps_len = 0)
{
    mfr_tuning t;
    const int st = resolve_tuning(tin, dtype, &t, rows == 1 && valid_dtype(dtype) ? (unsigned long long)cols * elem_size(dtype) : 0ull);
    if (st != MFR_OK) return st;
    const unsigned esize = elem_size(dtype);
    if (!out) return MFR_ERR_INVALID_ARG;
    if (rows > 0 && cols > 0 && !x) return MFR_ERR_INVALID_ARG;
    if (((size_t)x & (esize - 1u)) != 0) return MFR_ERR_INVALID_ARG;
    if (cols > ((size_t)1 << 60) || rows > ((size_t)1 << 40)) return MFR_ERR_INVALID_ARG;
    if (rows > 1 && row_stride < cols) return MFR_ERR_INVALID_ARG;
    if (!span_fits(rows, cols, row_stride)) return MFR_ERR_INVALID_ARG;
    if (rows == 0) return MFR_OK;
    resolve_load_policy(&t, rows * cols * esize);      // rows * cols <= the span < 2^60: no overflow

    int dev = 0;
    MFR_HIP(hipGetDevice(&dev));
    DeviceInfo info;
    const int ds = device_info(dev, &info);
    if (ds != MFR_OK) return ds;
    if (!info.gfx950) return MFR_ERR_UNSUPPORTED;

    if (cols == 0) return fill_zero(out, rows, stream);

    // Many rows: tiles shared out among rows, one launch for any alignment and stride.
    if (tin == nullptr) {
        mfr::RowsTiledShape shape;
        unsigned grid = 0;
        if (plan_rows_tiled((size_t)x, esize, rows, cols, row_stride, info.cus, &shape, &grid)) {
            const bool nt = t.nontemporal == 2;
            const hipError_t e =
                dtype == MFR_DTYPE_F16 ? mfr::launch_rows_tiled_f16(x, rows, cols, row_stride, out, shape, grid, nt, stream)
                : dtype == MFR_DTYPE_BF16 ? mfr::launch_rows_tiled_bf16(x, rows, cols, row_stride, out, shape, grid, nt, stream)
                                          : mfr::launch_rows_tiled_f32(x, rows, cols, row_stride, out, shape, grid, nt, stream);
            if (e != hipSuccess) return hip_fail(e, "rows_tiled launch");
            return MFR_OK;           // the few rows whose last 16-byte slot would reach past the array are summed by extra blocks of the same launch
        }
    }

    // Block size, blocks per row, chain shape, stagger of the per-row kernels for this call.
    Plan p;
    long long grid = 0;
    const int gs = per_row_geometry((size_t)x, esize, rows, cols, row_stride, tin == nullptr, info.cus, &t, &p, &grid);
    if (gs != MFR_OK) return gs;
    const size_t batch = rows < kMaxRowsPerLaunch ? rows : kMaxRowsPerLaunch;
    const bool two_launches = t.combine == MFR_COMBINE_TWO_LAUNCHES || grid > kSingleLaunchHardMax ||
                              (t.combine == MFR_COMBINE_AUTO && grid > kSingleLaunchAutoMax);
    if (stamps && stamps_len < 4u * (size_t)grid) return MFR_ERR_INVALID_ARG;
    p.a.stamps = stamps;
    ScratchView s;
    std::unique_lock<std::mutex> launch_lock;      // released when this call has enqueued its last kernel
    if (grid > 1) {
        // one float per block and row for the second launch to read, or one slot per block and row
        const size_t partial_count = two_launches ? (size_t)grid * batch : 1;
        const size_t slot_count = two_launches ? 1 : (size_t)grid * batch;
        if (fixed) {
            if (partial_count > fixed->partials_capacity || slot_count > fixed->slots_capacity) return MFR_ERR_SCRATCH_LIMIT;
            s = *fixed;
            launch_lock = std::unique_lock<std::mutex>(*fixed->launch_mutex);
        } else {
            const int ss = get_scratch(dev, stream, partial_count, slot_count, &s, &launch_lock);
            if (ss != MFR_OK) return ss;
        }
    }

    for (size_t r0 = 0; r0 < rows; r0 += batch) {
        const size_t nr = rows - r0 < batch ? rows - r0 : batch;
        const char *xr = (const char *)x + r0 * row_stride * esize;
        p.a.base = (const uint4v *)((size_t)xr & ~(size_t)15);
        p.a.x = xr;
        p.a.row_bytes = (unsigned long long)row_stride * esize;
        if (t.kernel == MFR_KERNEL_SPLIT) {
            // the same fraction of the chains and of the waves; a part without waves gets no chains
            const unsigned long long W = (unsigned long long)grid * (unsigned)p.waves;
            unsigned long long w1 = (W * (unsigned)t.split_permille + 500ull) / 1000ull;
            unsigned long long c1 = (p.a.chains * (unsigned)t.split_permille + 500ull) / 1000ull;
            if (w1 == 0) c1 = 0;
            if (w1 >= W) { w1 = W; c1 = p.a.chains; }
            if (c1 == 0) w1 = 0;
            if (c1 == p.a.chains) w1 = W;
            p.a.split_waves = w1;
            p.a.split_chains = c1;
        }
        p.a.partials = s.partials;
        p.a.combine_slots = two_launches ? nullptr : s.slots;
        p.a.out = out + r0;
        const hipError_t e = launch_dtype(dtype, p, dim3((unsigned)grid, (unsigned)nr), t, stream);
        if (e != hipSuccess) return hip_fail(e, "kernel launch");
        if (grid > 1 && two_launches) {
            hipLaunchKernelGGL(combine_kernel, dim3((unsigned)nr), dim3(grid > 4096 ? 1024 : 256), 0, stream,
                               (const float *)s.partials, (unsigned int)grid, out + r0);
            const hipError_t e2 = hipGetLastError();
            if (e2 != hipSuccess) return hip_fail(e2, "combine launch");
        }
    }
    return MFR_OK;
}

// Algorithm 1: relaunch the level kernel until one value is left.
int recurrence_impl(const mfr_half *x, size_t n, float *out, int R, hipStream_t stream)
{
    if (R < 1 || R > 8) return MFR_ERR_INVALID_ARG;
    if (!out) return MFR_ERR_INVALID_ARG;
    if (n > 0 && !x) return MFR_ERR_INVALID_ARG;
    if (((size_t)x & 1u) != 0 || n > ((size_t)1 << 60)) return MFR_ERR_INVALID_ARG;
    int dev = 0;
    MFR_HIP(hipGetDevice(&dev));
    DeviceInfo info;
    const int ds = device_info(dev, &info);
    if (ds != MFR_OK) return ds;
    if (!info.gfx950) return MFR_ERR_UNSUPPORTED;
    if (n == 0) return fill_zero(out, 1, stream);

    const size_t group = (size_t)R * 512;
    const size_t first = (n + 7 + group - 1) / group + 1;      // level-1 values (head padding included)
    const size_t second = (first + group - 1) / group + 1;
    const size_t first_padded = (first + 7) / 8 * 8;            // keeps the second buffer 16-byte aligned
    unsigned short *levels = nullptr;
    std::unique_lock<std::mutex> launch_lock;      // the levels of one call stay together in the stream
    {
        Scratch *entry = nullptr;
        {
            std::lock_guard<std::mutex> lock(g_mutex);
            entry = &g_scratch[std::make_pair(dev, stream)];
        }
        launch_lock = std::unique_lock<std::mutex>(entry->launch_mutex);
        std::lock_guard<std::mutex> lock(g_mutex);
        Scratch &s = *entry;
        const int st = grow((void **)&s.levels, &s.levels_capacity, first_padded + second + 8, sizeof(unsigned short),
                            4096, false, &s.retired);
        if (st != MFR_OK) return st;
        levels = s.levels;
    }
    unsigned short *buf[2] = {levels, levels + first_padded};

    const void *cur = x;
    size_t count = n;
    int k = 0;
    do {
        mfr::SumArgs a;
        memset(&a, 0, sizeof a);
        const unsigned head = (unsigned)(((size_t)cur & 15u) / 2u);
        a.base = (const uint4v *)((size_t)cur & ~(size_t)15);
        a.x = cur;
        a.n = count;
        a.head = head;
        a.vend = (unsigned long long)head + count;
        a.slots = (a.vend + 7ull) / 8ull;
        a.chains = (a.slots + 64ull * (unsigned)R - 1ull) / (64ull * (unsigned)R);   // groups, the last one padded
        const hipError_t e = mfr::launch_recurrence_level(a, R, buf[k & 1], a.chains == 1 ? out : nullptr, stream);
        if (e != hipSuccess) return hip_fail(e, "recurrence level launch");
        cur = buf[k & 1];
        count = (size_t)a.chains;
        ++k;
    } while (count > 1);
    return MFR_OK;
}

__global__ void store_zero_f64_kernel(double *out) { *out = 0.0; }

// fp16 input, chains in fp32, everything after a chain in binary64, double result.
int sum_wide_impl(const mfr_half *x, size_t n, double *out, const mfr_tuning *tin, hipStream_t stream)
{
    mfr_tuning in;
    memset(&in, 0, sizeof in);
    if (tin) in = *tin;
    if (in.chain_R == 0) in.chain_R = 1;          // shortest fp32 accumulation per column
    mfr_tuning t;
    const int st = resolve_tuning(&in, MFR_DTYPE_F16, &t);
    if (st != MFR_OK) return st;
    resolve_load_policy(&t, n * 2);
    if (t.kernel != MFR_KERNEL_MFMA || t.block_threads == 32) return MFR_ERR_INVALID_ARG;
    if (!out || ((size_t)out & 7u) != 0) return MFR_ERR_INVALID_ARG;
    if (n > 0 && !x) return MFR_ERR_INVALID_ARG;
    if (((size_t)x & 1u) != 0 || n > ((size_t)1 << 60)) return MFR_ERR_INVALID_ARG;
    int dev = 0;
    MFR_HIP(hipGetDevice(&dev));
    DeviceInfo info;
    const int ds = device_info(dev, &info);
    if (ds != MFR_OK) return ds;
    if (!info.gfx950) return MFR_ERR_UNSUPPORTED;
    if (n == 0) {
        hipLaunchKernelGGL(store_zero_f64_kernel, dim3(1), dim3(1), 0, stream, out);
        MFR_HIP(hipGetLastError());
        return MFR_OK;
    }
    Plan p;
    plan_region(n, (size_t)x, 2, t, &p);
    const long long grid = grid_blocks_for(p, t, info.cus, 1);
    if (grid < 1) return MFR_ERR_INVALID_ARG;
    const bool two_launches = t.combine == MFR_COMBINE_TWO_LAUNCHES || grid > kSingleLaunchHardMax ||
                              (t.combine == MFR_COMBINE_AUTO && grid > kSingleLaunchAutoMax);
    ScratchView s;
    std::unique_lock<std::mutex> launch_lock;
    if (grid > 1) {
        // binary64 partials and 64-bit slots: two words of the 4-byte arrays each (hipMalloc'ed: 8-byte aligned)
        const int ss = get_scratch(dev, stream, two_launches ? 2 * (size_t)grid + 2 : 1, two_launches ? 1 : 2 * (size_t)grid + 2,
                                   &s, &launch_lock);
        if (ss != MFR_OK) return ss;
    }
    p.a.base = (const uint4v *)((size_t)x & ~(size_t)15);
    p.a.x = x;
    p.a.partials = s.partials;
    p.a.combine_slots = two_launches ? nullptr : s.slots;
    p.a.out = (float *)out;
    const hipError_t e = mfr::launch_sum_wide(p, dim3((unsigned)grid), t, stream);
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    return MFR_OK;
}

int sum_impl(const void *x, int dtype, size_t n, float *out, const mfr_tuning *tin, hipStream_t stream)
{
    return sum_rows_impl(x, dtype, 1, n, n, out, tin, stream);
}

// Scratch of the entry point that allocates nothing: block partials (two-launch combine), then
// slots (single-launch combine), in a device array that every GPU the library runs on holds from
// the load of the code object to the end of the process.  Zero when loaded; the partials need no
// initial value and the reading block puts the zero back into every slot it has read.
constexpr size_t kStaticPartials = 8192;       // floats: grids of up to this many blocks
constexpr size_t kStaticSlots = 8192;          // words: the same
static __device__ __align__(256) unsigned char scratch[(kStaticPartials + kStaticSlots) * 4];

// The array's address on each device.  `scratch` itself is a host-side handle, not a device
// address: only what hipGetSymbolAddress returns for the current device may reach a kernel.
unsigned char *g_static_scratch[64];
std::mutex g_static_launch_mutex[64];      // one call's launches stay together (host threads sharing a stream)

int static_scratch(int dev, ScratchView *out)
{
    if (dev < 0 || dev >= 64) return MFR_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_static_scratch[dev]) {
        void *ptr = nullptr;
        MFR_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));     // for the current device, which is `dev`
        if (!ptr) return hip_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
        g_static_scratch[dev] = (unsigned char *)ptr;
    }
    out->partials = (float *)g_static_scratch[dev];
    out->partials_capacity = kStaticPartials;
    out->slots = (unsigned int *)(g_static_scratch[dev] + kStaticPartials * sizeof(float));
    out->slots_capacity = kStaticSlots;
    out->launch_mutex = &g_static_launch_mutex[dev];
    return MFR_OK;
}

}  // namespace

extern "C" {

int mfr_sum_f16(const mfr_half *x, size_t n, float *out, hipStream_t stream)
{
    return sum_impl(x, MFR_DTYPE_F16, n, out, nullptr, stream);
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
    return sum_impl(x, MFR_DTYPE_F16, n, out, &t, stream);
}

int mfr_sum_f16_ex(const mfr_half *x, size_t n, float *out, const mfr_tuning *t, hipStream_t stream)
{
    return sum_impl(x, MFR_DTYPE_F16, n, out, t, stream);
}

int mfr_sum_f16_noalloc(const mfr_half *x, size_t n, float *out, const mfr_tuning *t, hipStream_t stream)
{
    // argument errors first, as everywhere: they do not depend on a device being present
    mfr_tuning resolved;
    const int st = resolve_tuning(t, MFR_DTYPE_F16, &resolved);
    if (st != MFR_OK) return st;
    if (!out || (n > 0 && !x) || ((size_t)x & 1u) != 0) return MFR_ERR_INVALID_ARG;
    int dev = 0;
    MFR_HIP(hipGetDevice(&dev));
    ScratchView fixed;
    const int ss = static_scratch(dev, &fixed);
    if (ss != MFR_OK) return ss;
    return sum_rows_impl(x, MFR_DTYPE_F16, 1, n, n, out, t, stream, &fixed);
}

int mfr_sum_f16_stamped(const mfr_half *x, size_t n, float *out, const mfr_tuning *t, unsigned long long *stamps,
                        size_t stamps_len, hipStream_t stream)
{
    if (!stamps) return MFR_ERR_INVALID_ARG;
    return sum_rows_impl(x, MFR_DTYPE_F16, 1, n, n, out, t, stream, nullptr, stamps, stamps_len);
}

int mfr_wall_clock_khz(int *khz)
{
    if (!khz) return MFR_ERR_INVALID_ARG;
    int dev = 0;
    MFR_HIP(hipGetDevice(&dev));
    MFR_HIP(hipDeviceGetAttribute(khz, hipDeviceAttributeWallClockRate, dev));
    return MFR_OK;
}

int mfr_sum_bf16(const uint16_t *x, size_t n, float *out, hipStream_t stream)
{
    return sum_impl(x, MFR_DTYPE_BF16, n, out, nullptr, stream);
}

int mfr_sum_f32(const float *x, size_t n, float *out, hipStream_t stream)
{
    return sum_impl(x, MFR_DTYPE_F32, n, out, nullptr, stream);
}

int mfr_sum_ex(const void *x, int dtype, size_t n, float *out, const mfr_tuning *t, hipStream_t stream)
{
    return sum_impl(x, dtype, n, out, t, stream);
}

int mfr_sum_rows_ex(const void *x, int dtype, size_t rows, size_t cols, size_t row_stride, float *out,
                    const mfr_tuning *t, hipStream_t stream)
{
    return sum_rows_impl(x, dtype, rows, cols, row_stride, out, t, stream);
}

int mfr_sum_f16_rows(const mfr_half *x, size_t rows, size_t cols, size_t row_stride, float *out,
                     hipStream_t stream)
{
    return sum_rows_impl(x, MFR_DTYPE_F16, rows, cols, row_stride, out, nullptr, stream);
}

int mfr_sum_f16_f64(const mfr_half *x, size_t n, double *out, hipStream_t stream)
{
    return sum_wide_impl(x, n, out, nullptr, stream);
}

int mfr_sum_f16_f64_ex(const mfr_half *x, size_t n, double *out, const mfr_tuning *t, hipStream_t stream)
{
    return sum_wide_impl(x, n, out, t, stream);
}

int mfr_sum_f16_recurrence(const mfr_half *x, size_t n, float *out, int chain_R, hipStream_t stream)
{
    return recurrence_impl(x, n, out, chain_R, stream);
}

int mfr_get_default_tuning(int *block_threads, int *chain_R, int *grid_blocks)
{
    const DefaultGeometry &g = default_geometry();
    if (!g.valid) return MFR_ERR_INVALID_ARG;
    if (block_threads) *block_threads = g.block;
    if (chain_R) *chain_R = g.chain_R ? g.chain_R : kDefaultR;
    if (grid_blocks) *grid_blocks = MFR_GRID_AUTO;
    return MFR_OK;
}

long long mfr_grid_for(size_t n, size_t x_addr, const mfr_tuning *tin)
{
    mfr_tuning t;
    if (resolve_tuning(tin, MFR_DTYPE_F16, &t, (unsigned long long)n * 2ull) != MFR_OK) return -1;
    if (n == 0) return 1;
    Plan p;
    plan_region(n, x_addr, 2, t, &p);
    if (tin == nullptr && n * 2ull <= kMidSizeMinBytes && one_block_default(p.chains, &t)) return 1;
    int cus = 0;
    if (t.grid_blocks == MFR_GRID_AUTO) {
        int dev = 0;
        DeviceInfo info;
        if (hipGetDevice(&dev) != hipSuccess || device_info(dev, &info) != MFR_OK) return -1;
        cus = info.cus;
    }
    return grid_blocks_for(p, t, cus, 1);
}

int mfr_plan_ex(size_t n, size_t x_addr, int dtype, const mfr_tuning *tin, unsigned long long plan[7])
{
    mfr_tuning t;
    const int st = resolve_tuning(tin, dtype, &t, valid_dtype(dtype) ? (unsigned long long)n * elem_size(dtype) : 0ull);
    if (st != MFR_OK) return st;
    const unsigned esize = elem_size(dtype);
    if (!plan || (x_addr & (esize - 1u)) || n > ((size_t)1 << 60)) return MFR_ERR_INVALID_ARG;
    Plan p;
    plan_region(n, x_addr, esize, t, &p);
    plan[0] = p.a.head;
    plan[1] = p.a.slots;
    plan[2] = p.a.main0;
    plan[3] = p.a.chains;
    plan[4] = p.half ? 32ull : 64ull;
    plan[5] = p.a.epi0;
    plan[6] = p.a.epi1;
    return MFR_OK;
}

int mfr_plan_for(size_t n, size_t x_addr, const mfr_tuning *tin, unsigned long long plan[7])
{
    return mfr_plan_ex(n, x_addr, MFR_DTYPE_F16, tin, plan);
}

int mfr_rows_plan(size_t x_addr, int dtype, size_t rows, size_t cols, size_t row_stride, int cus,
                  unsigned long long plan[12])
{
    if (!valid_dtype(dtype) || !plan || cus < 1) return -MFR_ERR_INVALID_ARG;
    const unsigned esize = elem_size(dtype);
    if ((x_addr & (esize - 1u)) || cols > ((size_t)1 << 60) || rows > ((size_t)1 << 40)) return -MFR_ERR_INVALID_ARG;
    if (rows > 1 && row_stride < cols) return -MFR_ERR_INVALID_ARG;
    if (!span_fits(rows, cols, row_stride)) return -MFR_ERR_INVALID_ARG;
    mfr::RowsTiledShape s;
    unsigned grid = 0;
    if (!plan_rows_tiled(x_addr, esize, rows, cols, row_stride, cus, &s, &grid)) return 0;
    plan[0] = 1ull << s.log2_p;
    plan[1] = (unsigned long long)s.tiles_per_step;
    plan[2] = (unsigned long long)s.groups;
    plan[3] = s.iters;
    plan[4] = s.batches;
    plan[5] = 0;
    plan[6] = s.plain_hi;
    plan[7] = 0;
    plan[8] = s.row_hi;
    plan[9] = s.all_plain ? 1ull : 0ull;
    plan[10] = grid;
    plan[11] = (s.tail ? 1ull : 0ull) | (s.shift ? 2ull : 0ull) | ((unsigned long long)s.tail_log2_p << 2);
    return 1;
}

int mfr_rows_geometry(size_t x_addr, int dtype, size_t rows, size_t cols, size_t row_stride, const mfr_tuning *tin,
                      int cus, unsigned long long plan[8])
{
    if (!valid_dtype(dtype) || !plan || cus < 1) return -MFR_ERR_INVALID_ARG;
    const unsigned esize = elem_size(dtype);
    if ((x_addr & (esize - 1u)) || cols == 0 || rows == 0 || cols > ((size_t)1 << 60) || rows > ((size_t)1 << 40))
        return -MFR_ERR_INVALID_ARG;
    if (rows > 1 && row_stride < cols) return -MFR_ERR_INVALID_ARG;
    if (!span_fits(rows, cols, row_stride)) return -MFR_ERR_INVALID_ARG;
    mfr_tuning t;
    const int st = resolve_tuning(tin, dtype, &t, rows == 1 ? (unsigned long long)cols * esize : 0ull);
    if (st != MFR_OK) return -st;
    if (tin == nullptr) {
        mfr::RowsTiledShape shape;
        unsigned tiled_grid = 0;
        if (plan_rows_tiled(x_addr, esize, rows, cols, row_stride, cus, &shape, &tiled_grid)) return 0;
    }
    Plan p;
    long long grid = 0;
    const int gs = per_row_geometry(x_addr, esize, rows, cols, row_stride, tin == nullptr, cus, &t, &p, &grid);
    if (gs != MFR_OK) return -gs;
    plan[0] = (unsigned long long)t.block_threads;
    plan[1] = (unsigned long long)grid;
    plan[2] = (unsigned long long)t.chain_R;
    plan[3] = (unsigned long long)t.chains_in_flight;
    plan[4] = p.a.chains;
    plan[5] = p.a.rotate_bytes;
    plan[6] = p.dynamic_lds;
    plan[7] = p.a.per_row_phase;
    return 1;
}

int mfr_release_scratch(hipStream_t stream)
{
    int dev = 0;
    MFR_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mutex);
    const auto it = g_scratch.find(std::make_pair(dev, stream));
    if (it == g_scratch.end()) return MFR_OK;
    MFR_HIP(hipStreamSynchronize(stream));       // earlier calls on the stream may still be using it
    Scratch &s = it->second;
    hipError_t first = hipSuccess;
    std::vector<void *> all = s.retired;
    all.push_back(s.partials);
    all.push_back(s.slots);
    all.push_back(s.levels);
    for (void *mem : all) {
        if (!mem) continue;
        const hipError_t e = hipFree(mem);
        if (e != hipSuccess && first == hipSuccess) first = e;
    }
    g_scratch.erase(it);
    if (first != hipSuccess) return hip_fail(first, "hipFree(scratch)");
    return MFR_OK;
}

const char *mfr_strerror(int status)
{
    switch (status) {
    case MFR_OK: return "success";
    case MFR_ERR_INVALID_ARG: return "invalid argument";
    case MFR_ERR_UNSUPPORTED: return "unsupported device (gfx950 required)";
    case MFR_ERR_HIP: return "HIP runtime error";
    case MFR_ERR_SCRATCH_LIMIT: return "the call needs more scratch than the fixed scratch region holds";
    default: return "unknown status";
    }
}

const char *mfr_last_hip_error(void) { return g_hip_error; }

int mfr_version(void) { return 610; }

}  // extern "C"
