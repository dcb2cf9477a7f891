// C ABI of the AASD hot path: argument validation and kernel launches (see include/aasd.h).
// Validation touches no HIP API, so every error path can be exercised without a GPU.
#include "aasd.h"
#include "aasd_hooks.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdarg>
#include <cstdio>
#include <atomic>
#include <cstdlib>
#include <cstring>

#include "retrieve.hip.h"
#include "row_finish.hip.h"
#include "gumbel.hip.h"
#include "pool.hip.h"
#include "row_sweep.hip.h"
#include "tree.hip.h"
#include "verify_tail.hip.h"
#include "verify_topk.hip.h"

// Scratch memory of aasd_verify_static, one copy per GPU, zero when the library is loaded: 256 KiB of arrival
// counters (2048 lines of 128 bytes), then 4 MiB of partial results.  Host code reaches it only through the
// address that hipGetSymbolAddress returns for the current device: here the array's name is a handle, not a
// device address.
static __device__ __align__(256) unsigned char scratch[(256u << 10) + (4u << 20)];

namespace {

thread_local char g_err[512] = "";
// measurement and test hooks (aasd_hooks.h): all off unless a caller switches them on for its own thread
thread_local hipEvent_t g_sweep_start = nullptr, g_sweep_stop = nullptr;
thread_local hipEvent_t g_draw_start = nullptr, g_draw_stop = nullptr;
thread_local int g_plan_block = 0, g_plan_unroll = 0, g_plan_nseg = 0;   // 0 = the library picks

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

bool valid_dtype(int32_t dt) { return dt == AASD_F32 || dt == AASD_BF16; }
size_t elt_size(int32_t dt) { return dt == AASD_F32 ? 4 : 2; }

// Launch plan of the row sweep: threads per workgroup, 16-byte loads in flight per lane and
// buffer, and how many contiguous segments a row is cut into (one workgroup each).
// Measured on MI355X at V = 128256 bf16 (non-temporal loads): 256 threads x 2 loads is the fastest shape, or
// within 1 % of it, at every row count, for verification (6.9 TB/s at 36864 rows against 6.7 for 1024 x 2) and
// for alignment sampling (whose occupancy is LDS- and register-bound).  With few rows one workgroup per row
// cannot fill the GPU (a single workgroup streams at some 15-30 GB/s), so rows are cut into segments until
// there are several thousand workgroups.  aasd_hook_sweep_plan overrides the plan for the calling thread
// (tests force every compiled shape with it; it accepts compiled shapes only).
struct SweepPlan { int block, unroll, nseg, seg_vecs, npart; };

constexpr int64_t kSplitBelowRows = 8192;

SweepPlan plan_sweep(bool align, int64_t rows, int32_t V, int32_t dt)
{
    const int per_vec = dt == AASD_BF16 ? 8 : 4;
    const int nvec_max = V / per_vec > 0 ? V / per_vec : 1;
    SweepPlan pl{256, 2, 1, 0, 0};
    if (rows > 0 && rows < kSplitBelowRows) {
        const int64_t target = align ? 6144 : 8192;   // workgroups wanted (measured: 2048 alignment rows are fastest in 3 segments, 4608 verify rows in 2)
        const int64_t want = (target + rows - 1) / rows;
        const int by_len = nvec_max / (pl.block * 2) > 0 ? nvec_max / (pl.block * 2) : 1;  // >= 2 vectors per lane
        const int by_part = aasd::kMaxPartials / (pl.block / aasd::kWave);
        int n = (int)(want < by_len ? want : by_len);
        pl.nseg = n < by_part ? n : by_part;
    }
    if (align) {
        // The alignment sweep keeps one chunk maximum per 16-byte vector in LDS.  Rows are cut further until at
        // least four workgroups fit the 160 KB of a compute unit (V = 152064 bf16 needs 45 KB in one piece and runs
        // 4 % faster in two); a piece that cannot fit at all runs without the array.
        const size_t elt = dt == AASD_BF16 ? 2 : 4;
        const int by_part = aasd::kMaxPartials / (pl.block / aasd::kWave);
        while (pl.nseg < by_part) {
            const size_t per_lane = (size_t)((nvec_max + pl.nseg - 1) / pl.nseg + pl.block - 1) / pl.block * elt;
            const size_t stride = (per_lane + 15) / 16 * 16 + 16;
            if (stride * pl.block <= 40 * 1024) break;
            ++pl.nseg;
        }
    }
    if (g_plan_block > 0) { pl.block = g_plan_block; pl.unroll = g_plan_unroll; }
    if (g_plan_nseg > 0) pl.nseg = g_plan_nseg;
    const int waves = pl.block / aasd::kWave > 0 ? pl.block / aasd::kWave : 1;
    if (pl.nseg * waves > aasd::kMaxPartials) pl.nseg = aasd::kMaxPartials / waves > 0 ? aasd::kMaxPartials / waves : 1;
    const int per_seg = (nvec_max + pl.nseg - 1) / pl.nseg;
    pl.seg_vecs = (per_seg + pl.block - 1) / pl.block * pl.block;
    pl.npart = pl.nseg * waves;
    return pl;
}

// Plan of the tree-verification sweep.  The logits have room for max_nodes rows per tree, but a tree rarely fills its
// budget and the host does not know the counts, so the rows are cut as if a quarter of them were in use: a sparse
// batch then still has enough workgroups to fill the GPU (256 trees with 1695 of 24832 rows in use: 2 segments per
// row), and a full one only gets more, shorter workgroups, which a long launch does not feel.
SweepPlan plan_tree_sweep(int64_t rows, int32_t V, int32_t dt)
{
    return plan_sweep(false, rows >= 4 ? rows / 4 : 1, V, dt);
}

// Plan of the one-launch form of verification.  Its workgroups do not end with the sweep: each sends its partial
// to memory, waits, and is counted in (about a microsecond without loads in flight).  That costs nothing while
// all workgroups of the launch are on the GPU at once (it is paid once, at the end), so a short launch is cut into
// at most as many workgroups as the GPU holds at once: 256 compute units x the waves per SIMD that the kernel's
// registers allow (7 with 4 loads in flight per lane, 5 with 8, 4 with 16) x 4 SIMDs / waves per workgroup.
// More loads in flight did not make short launches faster (measured: 4, 8 and 16 within 2 %), so 4 it is.
int64_t fused_resident(int block, int unroll)
{
    const int waves_per_simd = unroll >= 4 ? 4 : (unroll == 2 ? 5 : 7);
    return (int64_t)256 * (waves_per_simd * 4 / (block / aasd::kWave));
}

SweepPlan plan_fused(int64_t rows, int32_t V, int32_t dt)
{
    SweepPlan pl = plan_sweep(false, rows, V, dt);
    if (g_plan_block == 0) pl.unroll = 1;   // the kernel keeps 4 x this many loads per lane in flight
    if (g_plan_nseg == 0 && rows > 0 && pl.nseg > 1) {
        const int64_t fit = fused_resident(pl.block, pl.unroll) / rows;
        const int nseg = (int)(fit < 1 ? 1 : (fit < pl.nseg ? fit : pl.nseg));
        if (nseg != pl.nseg) {
            const int per_vec = dt == AASD_BF16 ? 8 : 4;
            const int nvec_max = V / per_vec > 0 ? V / per_vec : 1;
            const int waves = pl.block / aasd::kWave;
            pl.nseg = nseg;
            pl.seg_vecs = ((nvec_max + nseg - 1) / nseg + pl.block - 1) / pl.block * pl.block;
            pl.npart = nseg * waves;
        }
    }
    return pl;
}

// Whether a verification with a zeroed counter area goes out as one launch.  One launch saves the host a launch
// (V = 128256 bf16, 9 rows, calls issued back to back: 10.6 us per call against 13.0); on the GPU the two kernels are
// by now as fast or faster (replayed from a graph: 9 rows 6.9 us in one launch, 6.7 in two; 288 rows 19.4 and 18.1),
// because the sweep kernel may cut rows into more and shorter workgroups than the GPU holds at once, which the
// one-launch form must not (its workgroups end with a trip to memory and an arrival, hidden only while they all run
// together; 8256 rows: 413 us against 397).  So the flag buys one launch where launches are what a call costs: up to
// 32 MiB of logits (128 rows at this V).
constexpr int64_t kOneLaunchMaxBytes = (int64_t)32 << 20;
bool takes_one_launch(int64_t rows, int32_t V, int32_t dt, const SweepPlan& pf)
{
    return rows * V * (int64_t)elt_size(dt) <= kOneLaunchMaxBytes && rows * pf.nseg <= fused_resident(pf.block, pf.unroll);
}

// the (threads, loads in flight) shapes the sweep kernels are compiled for
bool compiled_shape(int block, int unroll)
{
    return (block == 256 && (unroll == 1 || unroll == 2 || unroll == 4)) || (block == 512 && (unroll == 2 || unroll == 4)) ||
           (block == 1024 && (unroll == 1 || unroll == 2));
}

constexpr size_t kMaxChunkMaxLds = 60 * 1024;      // dynamic LDS the sweep may use for chunk maxima
constexpr int64_t kMaxUnitsPerLaunch = 1 << 22;    // keeps gridDim.x * blockDim.x below 2^32

// floor(2^32 / d) + 1: x / d = (x * magic) >> 32 for x < 2^32 / d (the kernels divide small unit and row indices so)
uint32_t div_magic(int32_t d) { return d > 1 ? (uint32_t)(((uint64_t)1 << 32) / (uint64_t)d + 1) : 0u; }

// A launch whose own begin and end are written to the hook's events, if any: the events then hold the kernel's
// duration as a profiler sees it, without the stream's gaps before and after it.
template <class Kernel, class... Args>
void launch_timed(Kernel kernel, dim3 grid, dim3 block, size_t lds, hipStream_t stream, hipEvent_t start, hipEvent_t stop, Args... args)
{
    if (start || stop) hipExtLaunchKernelGGL(kernel, grid, block, (unsigned)lds, stream, start, stop, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, lds, stream, args...);
}

template <int DT, bool ALIGN, bool COUNT, int BLOCK, int U>
hipError_t launch_sweep_one(const aasd::SweepParams& p, int64_t units, size_t dyn_lds, hipStream_t stream)
{
    const int64_t chunk = kMaxUnitsPerLaunch / p.nseg * p.nseg;   // whole rows per launch
    for (int64_t unit0 = 0; unit0 < units; unit0 += chunk) {
        const int64_t n = units - unit0 < chunk ? units - unit0 : chunk;
        launch_timed(aasd::row_sweep_kernel<DT, ALIGN, COUNT, BLOCK, U>, dim3((unsigned)n), dim3(BLOCK), dyn_lds, stream,
                     unit0 == 0 ? g_sweep_start : nullptr, unit0 + n >= units ? g_sweep_stop : nullptr, p, unit0 / p.nseg);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int DT, bool ALIGN, bool COUNT>
int launch_sweep(const aasd::SweepParams& p, const SweepPlan& pl, int64_t rows, size_t dyn_lds, hipStream_t stream)
{
    const int64_t units = rows * pl.nseg;
    hipError_t e;
    if (pl.block == 256 && pl.unroll == 4) e = launch_sweep_one<DT, ALIGN, COUNT, 256, 4>(p, units, dyn_lds, stream);
    else if (pl.block == 256 && pl.unroll == 2) e = launch_sweep_one<DT, ALIGN, COUNT, 256, 2>(p, units, dyn_lds, stream);
    else if (pl.block == 256 && pl.unroll == 1) e = launch_sweep_one<DT, ALIGN, COUNT, 256, 1>(p, units, dyn_lds, stream);
    else if (pl.block == 512 && pl.unroll == 4) e = launch_sweep_one<DT, ALIGN, COUNT, 512, 4>(p, units, dyn_lds, stream);
    else if (pl.block == 512 && pl.unroll == 2) e = launch_sweep_one<DT, ALIGN, COUNT, 512, 2>(p, units, dyn_lds, stream);
    else if (pl.block == 1024 && pl.unroll == 2) e = launch_sweep_one<DT, ALIGN, COUNT, 1024, 2>(p, units, dyn_lds, stream);
    else if (pl.block == 1024 && pl.unroll == 1) e = launch_sweep_one<DT, ALIGN, COUNT, 1024, 1>(p, units, dyn_lds, stream);
    else return fail(AASD_ERR_UNSUPPORTED, "sweep plan %d,%d is not a compiled launch shape", pl.block, pl.unroll);   // unreachable: plans are checked when set
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "row sweep launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

// Sweep and verification tail in one launch per chunk of units (verify_fused_kernel).
template <int DT, int BLOCK, int U>
hipError_t launch_fused_one(const aasd::VerifyFusedParams& p, int64_t units, hipStream_t stream)
{
    const int64_t chunk = kMaxUnitsPerLaunch / p.s.nseg * p.s.nseg;   // whole rows per launch
    for (int64_t unit0 = 0; unit0 < units; unit0 += chunk) {
        const int64_t n = units - unit0 < chunk ? units - unit0 : chunk;
        launch_timed(aasd::verify_fused_kernel<DT, BLOCK, U>, dim3((unsigned)n), dim3(BLOCK), 0, stream,
                     unit0 == 0 ? g_sweep_start : nullptr, unit0 + n >= units ? g_sweep_stop : nullptr, p, unit0 / p.s.nseg);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int DT>
int launch_fused(const aasd::VerifyFusedParams& p, const SweepPlan& pl, int64_t rows, hipStream_t stream)
{
    const int64_t units = rows * pl.nseg;
    hipError_t e;
    if (pl.block == 256 && pl.unroll == 4) e = launch_fused_one<DT, 256, 4>(p, units, stream);
    else if (pl.block == 256 && pl.unroll == 2) e = launch_fused_one<DT, 256, 2>(p, units, stream);
    else if (pl.block == 256 && pl.unroll == 1) e = launch_fused_one<DT, 256, 1>(p, units, stream);
    else if (pl.block == 512 && pl.unroll == 4) e = launch_fused_one<DT, 512, 4>(p, units, stream);
    else if (pl.block == 512 && pl.unroll == 2) e = launch_fused_one<DT, 512, 2>(p, units, stream);
    else if (pl.block == 1024 && pl.unroll == 2) e = launch_fused_one<DT, 1024, 2>(p, units, stream);
    else if (pl.block == 1024 && pl.unroll == 1) e = launch_fused_one<DT, 1024, 1>(p, units, stream);
    else return fail(AASD_ERR_UNSUPPORTED, "sweep plan %d,%d is not a compiled launch shape", pl.block, pl.unroll);   // unreachable
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "verify launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

// Sweep of the first rows_used[seq] rows of every sequence.  One launch covers `block` sequences; its grid is
// sized to the GPU, not to the input, or smaller if the rows cannot be that many.
template <int DT, int BLOCK, int U>
hipError_t launch_sweep_used_one(const aasd::SweepParams& p, const SweepPlan& pl, int64_t sequences, hipStream_t stream)
{
    // twice as many workgroups as the GPU holds at once (compute units x workgroups of this kernel per compute unit)
    static std::atomic<int64_t> cached{0};   // one GPU model per process: every thread would compute the same value
    int64_t resident = cached.load(std::memory_order_relaxed);
    if (resident == 0) {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, aasd::row_sweep_used_kernel<DT, BLOCK, U>, BLOCK, 0) != hipSuccess ||
            per_cu < 1)
            per_cu = 1;
        resident = (int64_t)cus * per_cu * 2;   // twice over: the second half starts as workgroups of the first end, which evens out their finish times
        cached.store(resident, std::memory_order_relaxed);
    }
    for (int64_t seq0 = 0; seq0 < sequences; seq0 += BLOCK) {
        const int nseq = (int)(sequences - seq0 < BLOCK ? sequences - seq0 : BLOCK);
        const int64_t most = (int64_t)nseq * p.rows_per_seq * pl.nseg;
        const unsigned grid = (unsigned)(most < resident ? most : resident);
        launch_timed(aasd::row_sweep_used_kernel<DT, BLOCK, U>, dim3(grid), dim3(BLOCK), 0, stream,
                     seq0 == 0 ? g_sweep_start : nullptr, seq0 + nseq >= sequences ? g_sweep_stop : nullptr, p, seq0, nseq);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int DT>
int launch_sweep_used(const aasd::SweepParams& p, const SweepPlan& pl, int64_t sequences, hipStream_t stream)
{
    hipError_t e;
    if (pl.block == 256 && pl.unroll == 4) e = launch_sweep_used_one<DT, 256, 4>(p, pl, sequences, stream);
    else if (pl.block == 256 && pl.unroll == 2) e = launch_sweep_used_one<DT, 256, 2>(p, pl, sequences, stream);
    else if (pl.block == 256 && pl.unroll == 1) e = launch_sweep_used_one<DT, 256, 1>(p, pl, sequences, stream);
    else if (pl.block == 512 && pl.unroll == 4) e = launch_sweep_used_one<DT, 512, 4>(p, pl, sequences, stream);
    else if (pl.block == 512 && pl.unroll == 2) e = launch_sweep_used_one<DT, 512, 2>(p, pl, sequences, stream);
    else if (pl.block == 1024 && pl.unroll == 2) e = launch_sweep_used_one<DT, 1024, 2>(p, pl, sequences, stream);
    else if (pl.block == 1024 && pl.unroll == 1) e = launch_sweep_used_one<DT, 1024, 1>(p, pl, sequences, stream);
    else return fail(AASD_ERR_UNSUPPORTED, "sweep plan %d,%d is not a compiled launch shape", pl.block, pl.unroll);   // unreachable
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "row sweep launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

template <int DT>
void launch_gumbel_dt(int m, unsigned grid, hipStream_t s, const aasd::GumbelParams& gp, int64_t u0, hipEvent_t start, hipEvent_t stop)
{
    const dim3 g(grid), b(aasd::kGumbelBlock);
    switch (m) {  // the kernel keeps m + 1 keys per lane
    case 1: launch_timed(aasd::gumbel_extras_kernel<DT, 2>, g, b, 0, s, start, stop, gp, u0); break;
    case 2: launch_timed(aasd::gumbel_extras_kernel<DT, 3>, g, b, 0, s, start, stop, gp, u0); break;
    case 3: launch_timed(aasd::gumbel_extras_kernel<DT, 4>, g, b, 0, s, start, stop, gp, u0); break;
    default: launch_timed(aasd::gumbel_extras_kernel<DT, 5>, g, b, 0, s, start, stop, gp, u0); break;
    }
}

void launch_gumbel(int32_t dt, int m, unsigned grid, hipStream_t s, const aasd::GumbelParams& gp, int64_t u0, hipEvent_t start, hipEvent_t stop)
{
    if (dt == AASD_BF16) launch_gumbel_dt<AASD_BF16>(m, grid, s, gp, u0, start, stop);
    else launch_gumbel_dt<AASD_F32>(m, grid, s, gp, u0, start, stop);
}

void launch_gumbel_merge(int m, int64_t rows, hipStream_t s, const aasd::GumbelParams& gp)
{
    const dim3 g((unsigned)((rows + aasd::kGumbelBlock - 1) / aasd::kGumbelBlock)), b(aasd::kGumbelBlock);
    switch (m) {
    case 1: hipLaunchKernelGGL((aasd::gumbel_merge_kernel<2>), g, b, 0, s, gp, rows); break;
    case 2: hipLaunchKernelGGL((aasd::gumbel_merge_kernel<3>), g, b, 0, s, gp, rows); break;
    case 3: hipLaunchKernelGGL((aasd::gumbel_merge_kernel<4>), g, b, 0, s, gp, rows); break;
    default: hipLaunchKernelGGL((aasd::gumbel_merge_kernel<5>), g, b, 0, s, gp, rows); break;
    }
}

size_t align16(size_t n) { return (n + 15) & ~(size_t)15; }

constexpr int32_t kMaxPoolCapacity = 1 << 24;

// Where the parts of a draft pool lie in the caller's buffer.
bool pool_layout(int32_t B, int32_t capacity, int32_t n_min, int32_t n_max, aasd::PoolLayout& lay, size_t& bytes)
{
    if (B < 0 || capacity < 1 || capacity > kMaxPoolCapacity || n_min < 1 || n_min > n_max || n_max > AASD_MAX_KEY) return false;
    const int NL = n_max - n_min + 1;
    int lg = 6;
    while (lg < 25 && ((int64_t)1 << lg) < 2 * ((int64_t)capacity + 1)) ++lg;   // load factor at most one half; a bucket has at most 25 bits
    lay.B = B; lay.capacity = capacity; lay.n_min = n_min; lay.n_max = n_max; lay.log2_table = lg;
    lay.counters = 0;
    lay.tables = align16((size_t)B * NL * sizeof(int32_t));
    lay.table_stride = align16((((size_t)1 << lg) + (size_t)capacity + 1) * sizeof(int32_t));
    bytes = lay.tables + (size_t)B * NL * lay.table_stride;
    return true;
}

// Workspace of aasd_verify: the arrival counters of the one-launch form (a 128-byte line each: one per sequence,
// plus one per group when a sequence's workgroups count in groups first), then the per-wave partial results of
// the sweep.
int verify_groups(int64_t rows, int64_t per_seq)
{
    // groups pay one more dependent atomic at the end of the launch; they are worth it only where a sequence's
    // workgroups all finish together (a short launch) and are many
    if (rows >= kSplitBelowRows || per_seq <= 24) return 1;
    int g = 1;
    while ((int64_t)g * g < per_seq) ++g;   // about sqrt(per_seq) groups of about sqrt(per_seq) workgroups
    return g;
}

size_t verify_counter_bytes(int32_t B, int ngroups)
{
    return (size_t)B * (size_t)(ngroups > 1 ? 1 + ngroups : 1) * aasd::kCounterWords * sizeof(unsigned);
}

// Layout of `scratch` and what the host keeps about it per GPU.
constexpr size_t kScratchCounterBytes = (size_t)256 << 10;
constexpr size_t kScratchPartialBytes = (size_t)4 << 20;
static_assert(sizeof(scratch) == kScratchCounterBytes + kScratchPartialBytes, "scratch layout");
constexpr int kMaxDevices = 64;
std::atomic<char*> g_scratch_ptr[kMaxDevices];    // device address of `scratch` on each GPU, once looked up
std::atomic<bool> g_scratch_dirty[kMaxDevices];   // a launch on it failed midway: its counters may not be zero

int verify_check(const void* logits, int32_t dt, int32_t B, int32_t C, int32_t k, int32_t V, int64_t row_stride,
                 int64_t seq_stride, const int32_t* drafts, const int32_t* draft_len, uint32_t flags,
                 const int32_t* accept_len, const int32_t* best_cand, const int32_t* next_token)
{
    if (!valid_dtype(dt)) return fail(AASD_ERR_INVALID_ARG, "verify: unknown dtype %d", dt);
    if (B < 0) return fail(AASD_ERR_INVALID_ARG, "verify: B = %d < 0", B);
    if (k < 1 || k > AASD_MAX_DRAFT) return fail(AASD_ERR_INVALID_ARG, "verify: k = %d outside [1,%d]", k, AASD_MAX_DRAFT);
    if (C < 1 || C > AASD_MAX_CANDIDATES) return fail(AASD_ERR_INVALID_ARG, "verify: C = %d outside [1,%d]", C, AASD_MAX_CANDIDATES);
    if (V <= 0) return fail(AASD_ERR_INVALID_ARG, "verify: V = %d <= 0", V);
    const int64_t R = 1 + (int64_t)C * k;
    if (row_stride < V) return fail(AASD_ERR_INVALID_ARG, "verify: row_stride %lld < V %d", (long long)row_stride, V);
    if (seq_stride < R * row_stride)
        return fail(AASD_ERR_INVALID_ARG, "verify: seq_stride %lld < R*row_stride %lld", (long long)seq_stride, (long long)(R * row_stride));
    if (flags & ~(AASD_VERIFY_NO_CLAMP | AASD_VERIFY_ZEROED_WORKSPACE)) return fail(AASD_ERR_INVALID_ARG, "verify: unknown flag bits 0x%x", flags);
    if (B == 0) return AASD_OK;
    if (!logits || !drafts || !draft_len || !accept_len || !best_cand || !next_token)
        return fail(AASD_ERR_INVALID_ARG, "verify: null required pointer");
    if (((uintptr_t)logits % elt_size(dt)) != 0)
        return fail(AASD_ERR_UNSUPPORTED, "verify: logits pointer is not aligned to its element size");
    return AASD_OK;
}

// The launches of conditional verification; every argument has been checked.  one_launch: sweep and tail in
// one kernel (the counters are zero); otherwise the sweep and then the tail kernel (the counters are not used).
int verify_launch(const void* logits, int32_t dt, int32_t B, int32_t C, int32_t k, int32_t V, int64_t row_stride,
                  int64_t seq_stride, const int32_t* drafts, const int32_t* draft_len, const uint8_t* strict, float alpha,
                  float beta, uint32_t flags, int32_t* accept_len, int32_t* best_cand, int32_t* next_token,
                  float* row_entropy, float* row_pmax, int32_t* row_argmax, float* tok_p, float* tok_delta,
                  uint32_t* near_count, unsigned* counters, void* partials, bool one_launch, hipStream_t s)
{
    const int64_t R = 1 + (int64_t)C * k;
    const int64_t rows = (int64_t)B * R;
    SweepPlan pl = plan_sweep(false, rows, V, dt);
    if (one_launch) {
        const SweepPlan pf = plan_fused(rows, V, dt);
        if (takes_one_launch(rows, V, dt, pf)) pl = pf;
        else one_launch = false;
    }
    aasd::SweepParams sp{};
    sp.logits = logits; sp.V = V; sp.row_stride = row_stride; sp.seq_stride = seq_stride; sp.rows_per_seq = (int32_t)R;
    sp.c = 1; sp.nseg = pl.nseg; sp.nseg_magic = div_magic(pl.nseg); sp.seg_vecs = pl.seg_vecs; sp.partials = (aasd::WavePartial*)partials;

    aasd::VerifyTailParams tp{};
    tp.logits = logits; tp.B = B; tp.C = C; tp.k = k; tp.V = V; tp.row_stride = row_stride; tp.seq_stride = seq_stride;
    tp.drafts = drafts; tp.draft_len = draft_len; tp.strict = strict; tp.alpha = alpha; tp.beta = beta;
    tp.flags = flags & AASD_VERIFY_NO_CLAMP;
    tp.accept_len = accept_len; tp.best_cand = best_cand; tp.next_token = next_token;
    tp.tok_p = tok_p; tp.tok_delta = tok_delta; tp.near_count = near_count;
    tp.row_entropy = row_entropy; tp.row_pmax = row_pmax; tp.row_argmax = row_argmax;
    tp.partials = (const aasd::WavePartial*)partials; tp.npart = pl.npart;

    if (one_launch) {
        aasd::VerifyFusedParams fp{};
        fp.s = sp; fp.t = tp; fp.counters = counters; fp.ngroups = verify_groups(rows, R * pl.nseg);
        fp.t.npart = pl.nseg;   // this form leaves one partial per workgroup, not per wave
        fp.rps_magic = div_magic((int32_t)R);   // R >= 2
        return dt == AASD_BF16 ? launch_fused<AASD_BF16>(fp, pl, rows, s) : launch_fused<AASD_F32>(fp, pl, rows, s);
    }
    if (pl.nseg >= 8 && pl.block > aasd::kWave) {
        // a short launch cut into many segments: one partial per workgroup instead of one per wave (up to 64 per row
        // otherwise), so that the tail merges a sequence's rows in one pass
        sp.merge_waves = 1;
        tp.npart = pl.nseg;
    }
    const int rc = dt == AASD_BF16 ? launch_sweep<AASD_BF16, false, false>(sp, pl, rows, 0, s)
                                   : launch_sweep<AASD_F32, false, false>(sp, pl, rows, 0, s);
    if (rc != AASD_OK) return rc;
    if (dt == AASD_BF16)
        hipLaunchKernelGGL(aasd::verify_tail_kernel<AASD_BF16>, dim3((unsigned)B), dim3(aasd::kTailBlock), 0, s, tp);
    else
        hipLaunchKernelGGL(aasd::verify_tail_kernel<AASD_F32>, dim3((unsigned)B), dim3(aasd::kTailBlock), 0, s, tp);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "verify tail launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

}  // namespace

extern "C" {

const char* aasd_version(void) { return "aasd-mi355x 0.1 (gfx950)"; }

const char* aasd_last_error(void) { return g_err; }

void aasd_hook_sweep_events(void* start, void* stop)
{
    g_sweep_start = (hipEvent_t)start;
    g_sweep_stop = (hipEvent_t)stop;
}

int aasd_hook_verify_launches(int32_t B, int32_t C, int32_t k, int32_t V, int32_t dt, uint32_t flags)
{
    if (B < 1 || C < 1 || C > AASD_MAX_CANDIDATES || k < 1 || k > AASD_MAX_DRAFT || V <= 0 || !valid_dtype(dt)) return 0;
    const int64_t rows = (int64_t)B * (1 + (int64_t)C * k);
    return (flags & AASD_VERIFY_ZEROED_WORKSPACE) && takes_one_launch(rows, V, dt, plan_fused(rows, V, dt)) ? 1 : 2;
}

void aasd_hook_draw_events(void* start, void* stop)
{
    g_draw_start = (hipEvent_t)start;
    g_draw_stop = (hipEvent_t)stop;
}

int aasd_hook_sweep_plan(int32_t threads, int32_t loads, int32_t segments)
{
    if (threads == 0 && loads == 0 && segments == 0) {
        g_plan_block = g_plan_unroll = g_plan_nseg = 0;
        return AASD_OK;
    }
    if (threads == 0 && loads == 0) {   // segments only
        if (segments < 1 || segments > 16) return fail(AASD_ERR_INVALID_ARG, "sweep plan: segments = %d outside [1,16]", segments);
        g_plan_block = g_plan_unroll = 0;
        g_plan_nseg = segments;
        return AASD_OK;
    }
    if (!compiled_shape(threads, loads))
        return fail(AASD_ERR_UNSUPPORTED, "sweep plan: %d threads x %d loads is not a compiled launch shape", threads, loads);
    if (segments < 0 || segments > 16) return fail(AASD_ERR_INVALID_ARG, "sweep plan: segments = %d outside [0,16]", segments);
    g_plan_block = threads; g_plan_unroll = loads; g_plan_nseg = segments;
    return AASD_OK;
}

size_t aasd_align_sample_workspace_bytes(int64_t rows, int32_t V, int32_t dt)
{
    if (rows < 0 || V <= 0 || !valid_dtype(dt)) return 0;
    const SweepPlan pl = plan_sweep(true, rows, V, dt);
    return (size_t)rows * pl.npart * (sizeof(aasd::WavePartial) + aasd::kListCap * sizeof(int32_t));
}

int aasd_align_sample(const void* logits, int32_t dt, int64_t rows, int32_t V, int64_t row_stride,
                      const int32_t* next_tok, int32_t m, int32_t c, int32_t mode, uint64_t seed,
                      uint64_t row_id_base, int32_t* argmax, uint8_t* misaligned, float* entropy,
                      float* p_next, float* p_max, int32_t* rank, int32_t* extras,
                      uint8_t* n_extras, uint32_t* near_count, void* workspace, size_t workspace_bytes,
                      void* stream)
{
    if (!valid_dtype(dt)) return fail(AASD_ERR_INVALID_ARG, "align_sample: unknown dtype %d", dt);
    if (rows < 0) return fail(AASD_ERR_INVALID_ARG, "align_sample: rows = %lld < 0", (long long)rows);
    if (V <= 0) return fail(AASD_ERR_INVALID_ARG, "align_sample: V = %d <= 0", V);
    if (row_stride < V) return fail(AASD_ERR_INVALID_ARG, "align_sample: row_stride %lld < V %d", (long long)row_stride, V);
    if (m < 0 || m > AASD_MAX_EXTRAS) return fail(AASD_ERR_INVALID_ARG, "align_sample: m = %d outside [0,%d]", m, AASD_MAX_EXTRAS);
    if (c < 1 || c < m || c > AASD_MAX_CANDSET)
        return fail(AASD_ERR_INVALID_ARG, "align_sample: c = %d outside [max(m,1),%d]", c, AASD_MAX_CANDSET);
    if (mode != AASD_EXTRAS_TOP && mode != AASD_EXTRAS_SAMPLE && mode != AASD_EXTRAS_GUMBEL)
        return fail(AASD_ERR_INVALID_ARG, "align_sample: unknown mode %d", mode);
    if (rows == 0) return AASD_OK;
    if (!logits || !argmax || !misaligned || !entropy || !p_next || !p_max)
        return fail(AASD_ERR_INVALID_ARG, "align_sample: null required pointer");
    if (m > 0 && (!extras || !n_extras))
        return fail(AASD_ERR_INVALID_ARG, "align_sample: extras and n_extras are required when m > 0");
    if (((uintptr_t)logits % elt_size(dt)) != 0)
        return fail(AASD_ERR_UNSUPPORTED, "align_sample: logits pointer is not aligned to its element size");
    const size_t need_ws = aasd_align_sample_workspace_bytes(rows, V, dt);
    if (!workspace || workspace_bytes < need_ws)
        return fail(AASD_ERR_WORKSPACE, "align_sample: workspace of %zu bytes needed, %zu given", need_ws,
                    workspace ? workspace_bytes : (size_t)0);
    if (((uintptr_t)workspace % 16) != 0) return fail(AASD_ERR_WORKSPACE, "align_sample: workspace is not 16-byte aligned");

    const SweepPlan pl = plan_sweep(true, rows, V, dt);
    aasd::WavePartial* partials = (aasd::WavePartial*)workspace;
    int32_t* lists = (int32_t*)((char*)workspace + (size_t)rows * pl.npart * sizeof(aasd::WavePartial));
    // full-vocabulary draws are made by a pass of their own over the misaligned rows: the statistics pass
    // then has no candidates to collect
    const bool gumbel = mode == AASD_EXTRAS_GUMBEL && m > 0;
    const int32_t m_draw = m;
    if (gumbel) m = 0;

    aasd::SweepParams p{};
    p.logits = logits; p.V = V; p.row_stride = row_stride; p.seq_stride = row_stride; p.rows_per_seq = 1;
    p.next_tok = next_tok; p.want_cand = m > 0; p.c = c;
    p.nseg = pl.nseg; p.nseg_magic = div_magic(pl.nseg); p.seg_vecs = pl.seg_vecs; p.partials = partials; p.lists = lists;
    // one chunk maximum per 16-byte vector of a segment, kept in LDS (lane-contiguous) when it fits
    size_t dyn = 0;
    if (m > 0 && next_tok) {
        const size_t per_lane = (size_t)(pl.seg_vecs / pl.block) * elt_size(dt);
        size_t stride = (per_lane + 15) / 16 * 16;  // 16-byte slots; an odd number of them spreads lanes over the banks
        if ((stride / 16) % 2 == 0) stride += 16;
        if (stride * pl.block <= kMaxChunkMaxLds) { dyn = stride * pl.block; p.cm_enabled = 1; p.cm_stride = (int32_t)stride; }
    }
    hipStream_t s = (hipStream_t)stream;
    int rc;
    if (dt == AASD_BF16)
        rc = rank ? launch_sweep<AASD_BF16, true, true>(p, pl, rows, dyn, s) : launch_sweep<AASD_BF16, true, false>(p, pl, rows, dyn, s);
    else
        rc = rank ? launch_sweep<AASD_F32, true, true>(p, pl, rows, dyn, s) : launch_sweep<AASD_F32, true, false>(p, pl, rows, dyn, s);
    if (rc != AASD_OK) return rc;

    aasd::AlignFinishParams f{};
    f.logits = logits; f.V = V; f.row_stride = row_stride; f.rows = rows; f.next_tok = next_tok;
    f.m_x = m; f.c = c; f.mode = mode; f.seed = seed; f.row_id_base = row_id_base;
    f.argmax = argmax; f.misaligned = misaligned; f.entropy = entropy; f.p_next = p_next; f.p_max = p_max;
    f.rank = rank; f.extras = extras; f.n_extras = n_extras; f.near_count = near_count;
    f.partials = partials; f.lists = lists; f.npart = pl.npart;
    const int rows_per_block = aasd::kFinishBlock / aasd::kWave;
    for (int64_t r0 = 0; r0 < rows; r0 += kMaxUnitsPerLaunch) {
        const int64_t n = rows - r0 < kMaxUnitsPerLaunch ? rows - r0 : kMaxUnitsPerLaunch;
        aasd::AlignFinishParams fc = f;
        // a chunk of rows: shift every per-row pointer
        fc.logits = (const char*)logits + (size_t)r0 * (size_t)row_stride * elt_size(dt);
        fc.rows = n; fc.row_id_base = row_id_base + (uint64_t)r0;
        fc.next_tok = next_tok ? next_tok + r0 : nullptr;
        fc.argmax = argmax + r0; fc.misaligned = misaligned + r0; fc.entropy = entropy + r0;
        fc.p_next = p_next + r0; fc.p_max = p_max + r0; fc.rank = rank ? rank + r0 : nullptr;
        fc.extras = extras ? extras + r0 * m : nullptr; fc.n_extras = n_extras ? n_extras + r0 : nullptr;
        fc.partials = partials + r0 * pl.npart; fc.lists = lists + r0 * pl.npart * aasd::kListCap;
        const unsigned grid = (unsigned)((n + rows_per_block - 1) / rows_per_block);
        if (dt == AASD_BF16) hipLaunchKernelGGL(aasd::align_finish_kernel<AASD_BF16>, dim3(grid), dim3(aasd::kFinishBlock), 0, s, fc);
        else hipLaunchKernelGGL(aasd::align_finish_kernel<AASD_F32>, dim3(grid), dim3(aasd::kFinishBlock), 0, s, fc);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "align finish launch failed: %s", hipGetErrorString(e));
    }
    if (gumbel) {
        aasd::GumbelParams gp{};
        gp.logits = logits; gp.V = V; gp.row_stride = row_stride; gp.next_tok = next_tok; gp.misaligned = misaligned;
        gp.m_x = m_draw; gp.seed = seed; gp.row_id_base = row_id_base;
        gp.extras = extras; gp.n_extras = n_extras; gp.extra_keys = nullptr; gp.near_count = near_count;
        // several workgroups per row while the rows are few; their best keys go through the workspace, which the
        // finish kernel no longer needs (at least 896 bytes per row; 16 shares x 5 keys need 640)
        int64_t nseg = (8192 + rows - 1) / rows;
        const int64_t nquad = ((int64_t)V + 3) / 4;
        if (nseg > 16) nseg = 16;
        if (nseg > nquad / aasd::kGumbelBlock) nseg = nquad / aasd::kGumbelBlock;
        if (g_plan_nseg > 0 && g_plan_nseg < nseg) nseg = g_plan_nseg;   // the hook's segment count also caps the shares per row
        if (nseg < 1) nseg = 1;
        gp.nseg = (int32_t)nseg;
        gp.part_z = (float*)workspace;
        gp.part_i = (int32_t*)((char*)workspace + align16((size_t)rows * nseg * (m_draw + 1) * sizeof(float)));
        const int64_t units = rows * nseg;
        for (int64_t u0 = 0; u0 < units; u0 += kMaxUnitsPerLaunch) {
            const int64_t n = units - u0 < kMaxUnitsPerLaunch ? units - u0 : kMaxUnitsPerLaunch;
            launch_gumbel(dt, m_draw, (unsigned)n, s, gp, u0, u0 == 0 ? g_draw_start : nullptr, u0 + n >= units ? g_draw_stop : nullptr);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "gumbel extras launch failed: %s", hipGetErrorString(e));
        }
        launch_gumbel_merge(m_draw, rows, s, gp);
        {
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "gumbel merge launch failed: %s", hipGetErrorString(e));
        }
    }
    return AASD_OK;
}

int aasd_retrieve_drafts(const int32_t* tokens, int64_t tok_stride, const int32_t* len,
                         const int32_t* prompt_len, int32_t B, int32_t n_min, int32_t n_max,
                         int32_t k, int32_t C, const int32_t* extras, const uint8_t* n_extras,
                         int32_t m, int64_t extras_stride, int32_t* drafts, int32_t* draft_len,
                         int32_t* src_pos, int32_t* n_cand, int32_t* key_len,
                         int32_t* draft_extras, uint8_t* strict, void* stream)
{
    if (B < 0) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: B = %d < 0", B);
    if (tok_stride < 1) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: tok_stride = %lld < 1", (long long)tok_stride);
    if (tok_stride > 0x7fffffffLL) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: tok_stride exceeds int32");
    if (n_min < 1 || n_min > n_max || n_max > AASD_MAX_KEY)
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: need 1 <= n_min <= n_max <= %d (got %d, %d)", AASD_MAX_KEY, n_min, n_max);
    if (k < 1 || k > AASD_MAX_DRAFT) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: k = %d outside [1,%d]", k, AASD_MAX_DRAFT);
    if (C < 1 || C > AASD_MAX_CANDIDATES)
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: C = %d outside [1,%d]", C, AASD_MAX_CANDIDATES);
    const bool have_table = extras != nullptr || n_extras != nullptr;
    if (have_table && (!extras || !n_extras))
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: extras and n_extras must be given together");
    if (have_table && (m < 1 || m > AASD_MAX_EXTRAS))
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: m = %d outside [1,%d] with an alignment table", m, AASD_MAX_EXTRAS);
    if (have_table && extras_stride < 0) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: extras_stride < 0");
    if (draft_extras && !have_table)
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: draft_extras needs the alignment table");
    if (B == 0) return AASD_OK;
    if (!tokens || !len || !prompt_len || !drafts || !draft_len || !src_pos || !n_cand || !key_len || !strict)
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: null required pointer");

    aasd::RetrieveParams p{};
    p.tokens = tokens; p.tok_stride = tok_stride; p.len = len; p.prompt_len = prompt_len;
    p.B = B; p.n_min = n_min; p.n_max = n_max; p.k = k; p.C = C;
    p.extras = extras; p.n_extras = n_extras; p.m_x = have_table ? m : 0; p.extras_stride = extras_stride;
    p.drafts = drafts; p.draft_len = draft_len; p.src_pos = src_pos; p.n_cand = n_cand; p.key_len = key_len;
    p.draft_extras = draft_extras; p.strict = strict;
    // Up to 512 sequences: 1024 threads each (all resident at once, the shortest chain of work per thread) and the
    // whole buffer in one LDS tile if it fits in 56 KB.  More sequences: 256 threads each, so that a compute unit holds several sequences at once and their load,
    // barrier and hash phases overlap (8192 sequences of 4352 tokens: 61 us against 145 us); one tile if the buffer
    // fits in 45 KB (a second tile costs more than the lower occupancy), else tiles of 22 KB.  Positions per lane
    // per tile are odd.
    const bool many = B > 512;   // more sequences than 1024-thread workgroups fit the GPU at once (2 per compute unit)
    const int block = many ? aasd::kRetrieveBlockSmall : aasd::kRetrieveBlock;
    int max_run = 11;
    if (many) max_run = (tok_stride + block - 1) / block <= 35 ? 35 : 17;   // (8 + 256*17) * 5 = 21,800 bytes; (8 + 1024*11) * 4 + 1024*11 = 56,352 bytes
    int run = (int)((tok_stride + block - 1) / block);
    if (run > max_run) run = max_run;
    run |= 1;
    p.run = run;
    p.tile = run * block;
    const size_t dyn = (size_t)(AASD_MAX_KEY + p.tile) * 4 + (size_t)p.tile;
    if (many) hipLaunchKernelGGL(aasd::retrieve_kernel<aasd::kRetrieveBlockSmall>, dim3((unsigned)B), dim3(block), dyn, (hipStream_t)stream, p);
    else hipLaunchKernelGGL(aasd::retrieve_kernel<aasd::kRetrieveBlock>, dim3((unsigned)B), dim3(block), dyn, (hipStream_t)stream, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "retrieve_drafts launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

size_t aasd_verify_workspace_bytes(int32_t B, int32_t C, int32_t k, int32_t V, int32_t dt)
{
    if (B < 0 || C < 1 || C > AASD_MAX_CANDIDATES || k < 1 || k > AASD_MAX_DRAFT || V <= 0 || !valid_dtype(dt)) return 0;
    const int64_t rows = (int64_t)B * (1 + C * k);
    const SweepPlan pl = plan_sweep(false, rows, V, dt);   // the two-launch form needs the most partials (one per wave)
    const SweepPlan pf = plan_fused(rows, V, dt);
    return verify_counter_bytes(B, verify_groups(rows, (int64_t)(1 + C * k) * pf.nseg)) + (size_t)rows * pl.npart * sizeof(aasd::WavePartial);
}

int aasd_verify(const void* logits, int32_t dt, int32_t B, int32_t C, int32_t k, int32_t V,
                int64_t row_stride, int64_t seq_stride, const int32_t* drafts,
                const int32_t* draft_len, const uint8_t* strict, float alpha, float beta,
                uint32_t flags, int32_t* accept_len, int32_t* best_cand, int32_t* next_token,
                float* row_entropy, float* row_pmax, int32_t* row_argmax, float* tok_p,
                float* tok_delta, uint32_t* near_count, void* workspace, size_t workspace_bytes,
                void* stream)
{
    const int rc = verify_check(logits, dt, B, C, k, V, row_stride, seq_stride, drafts, draft_len, flags, accept_len,
                                best_cand, next_token);
    if (rc != AASD_OK || B == 0) return rc;
    const size_t need = aasd_verify_workspace_bytes(B, C, k, V, dt);
    if (!workspace || workspace_bytes < need)
        return fail(AASD_ERR_WORKSPACE, "verify: workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
    if (((uintptr_t)workspace % 128) != 0) return fail(AASD_ERR_WORKSPACE, "verify: workspace is not 128-byte aligned");
    const size_t partial_bytes = (size_t)B * (1 + C * k) * plan_sweep(false, (int64_t)B * (1 + C * k), V, dt).npart * sizeof(aasd::WavePartial);
    return verify_launch(logits, dt, B, C, k, V, row_stride, seq_stride, drafts, draft_len, strict, alpha, beta, flags,
                         accept_len, best_cand, next_token, row_entropy, row_pmax, row_argmax, tok_p, tok_delta,
                         near_count, (unsigned*)workspace, (char*)workspace + (need - partial_bytes),
                         (flags & AASD_VERIFY_ZEROED_WORKSPACE) != 0, (hipStream_t)stream);
}

size_t aasd_verify_static_max_bytes(void) { return kScratchPartialBytes; }

int aasd_verify_static(const void* logits, int32_t dt, int32_t B, int32_t C, int32_t k, int32_t V,
                       int64_t row_stride, int64_t seq_stride, const int32_t* drafts,
                       const int32_t* draft_len, const uint8_t* strict, float alpha, float beta,
                       uint32_t flags, int32_t* accept_len, int32_t* best_cand, int32_t* next_token,
                       float* row_entropy, float* row_pmax, int32_t* row_argmax, float* tok_p,
                       float* tok_delta, uint32_t* near_count, void* stream)
{
    if (flags & AASD_VERIFY_ZEROED_WORKSPACE) return fail(AASD_ERR_INVALID_ARG, "verify_static: AASD_VERIFY_ZEROED_WORKSPACE is about a caller's workspace");
    const int rc = verify_check(logits, dt, B, C, k, V, row_stride, seq_stride, drafts, draft_len, flags, accept_len,
                                best_cand, next_token);
    if (rc != AASD_OK || B == 0) return rc;
    const int64_t R = 1 + (int64_t)C * k, rows = (int64_t)B * R;
    const size_t need = (size_t)rows * plan_sweep(false, rows, V, dt).npart * sizeof(aasd::WavePartial);
    if (need > kScratchPartialBytes)
        return fail(AASD_ERR_UNSUPPORTED, "verify_static: %zu bytes of partial results needed for %lld rows, the built-in scratch holds %zu "
                    "(use aasd_verify with a workspace)", need, (long long)rows, kScratchPartialBytes);
    // one launch only if its counters fit the built-in ones (they do for every shape that is served in one launch by
    // aasd_verify, which are decode steps of at most 1792 workgroups; checked all the same)
    const SweepPlan pf = plan_fused(rows, V, dt);
    const bool one_launch = verify_counter_bytes(B, verify_groups(rows, R * pf.nseg)) <= kScratchCounterBytes;

    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return fail(AASD_ERR_UNSUPPORTED, "verify_static: no current device, or its index is beyond %d", kMaxDevices - 1);
    char* base = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!base) {   // first call on this GPU: where its copy of the array lives
        void* sym = nullptr;
        const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !sym) return fail(AASD_ERR_LAUNCH, "verify_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
        base = (char*)sym;
        g_scratch_ptr[dev].store(base, std::memory_order_release);
    }
    hipStream_t s = (hipStream_t)stream;
    unsigned* counters = (unsigned*)base;
    if (one_launch && g_scratch_dirty[dev].exchange(false)) {
        // The counters are zero when the library is loaded and every completed call leaves them so; only a call
        // that failed between its launches can have left some behind.  (A fill kernel, not a memset: the caller may
        // be capturing a graph.)
        const int words = (int)(kScratchCounterBytes / sizeof(unsigned));
        hipLaunchKernelGGL(aasd::fill_u32_kernel, dim3((words + 255) / 256), dim3(256), 0, s, counters, 0u, words);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            g_scratch_dirty[dev].store(true);
            return fail(AASD_ERR_LAUNCH, "verify_static: clearing the counters failed: %s", hipGetErrorString(e));
        }
    }
    const int rc2 = verify_launch(logits, dt, B, C, k, V, row_stride, seq_stride, drafts, draft_len, strict, alpha, beta, flags,
                                  accept_len, best_cand, next_token, row_entropy, row_pmax, row_argmax, tok_p, tok_delta,
                                  near_count, counters, base + kScratchCounterBytes, one_launch, s);
    if (rc2 != AASD_OK) g_scratch_dirty[dev].store(true);
    return rc2;
}

size_t aasd_pool_bytes(int32_t B, int32_t capacity, int32_t n_min, int32_t n_max)
{
    aasd::PoolLayout lay;
    size_t bytes = 0;
    return pool_layout(B, capacity, n_min, n_max, lay, bytes) ? bytes : 0;
}

int aasd_pool_update(void* pool, size_t pool_bytes, int32_t B, int32_t capacity, int32_t n_min, int32_t n_max,
                     const int32_t* tokens, int64_t tok_stride, const int32_t* len, int32_t reset, void* stream)
{
    aasd::PoolLayout lay;
    size_t need = 0;
    if (!pool_layout(B, capacity, n_min, n_max, lay, need))
        return fail(AASD_ERR_INVALID_ARG, "pool_update: need B >= 0, 1 <= capacity <= %d, 1 <= n_min <= n_max <= %d (got %d, %d, %d, %d)",
                    kMaxPoolCapacity, AASD_MAX_KEY, B, capacity, n_min, n_max);
    if (tok_stride < 1 || tok_stride > 0x7fffffffLL) return fail(AASD_ERR_INVALID_ARG, "pool_update: tok_stride = %lld out of range", (long long)tok_stride);
    if (B == 0) return AASD_OK;
    if (!tokens || !len) return fail(AASD_ERR_INVALID_ARG, "pool_update: null required pointer");
    if (!pool || pool_bytes < need)
        return fail(AASD_ERR_WORKSPACE, "pool_update: pool of %zu bytes needed, %zu given", need, pool ? pool_bytes : (size_t)0);
    if (((uintptr_t)pool % 16) != 0) return fail(AASD_ERR_WORKSPACE, "pool_update: pool is not 16-byte aligned");
    aasd::PoolUpdateParams q{};
    q.pool = (char*)pool; q.lay = lay; q.tokens = tokens; q.tok_stride = tok_stride; q.len = len; q.reset = reset ? 1 : 0;
    const int64_t grid = (int64_t)B * (n_max - n_min + 1);
    if (grid > kMaxUnitsPerLaunch) return fail(AASD_ERR_UNSUPPORTED, "pool_update: too many sequences for one launch");
    hipLaunchKernelGGL(aasd::pool_build_kernel, dim3((unsigned)grid), dim3(aasd::kPoolBuildBlock), 0, (hipStream_t)stream, q);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "pool_update launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

static int pool_lookup(bool update_first, const void* pool, size_t pool_bytes, int32_t B, int32_t capacity, int32_t n_min,
                       int32_t n_max, const int32_t* tokens, int64_t tok_stride, const int32_t* len,
                       const int32_t* prompt_len, int32_t k, int32_t C, const int32_t* extras, const uint8_t* n_extras,
                       int32_t m, int64_t extras_stride, int32_t* drafts, int32_t* draft_len, int32_t* src_pos,
                       int32_t* n_cand, int32_t* key_len, int32_t* draft_extras, uint8_t* strict, void* stream)
{
    aasd::PoolLayout lay;
    size_t need = 0;
    if (!pool_layout(B, capacity, n_min, n_max, lay, need))
        return fail(AASD_ERR_INVALID_ARG, "pool_retrieve: need B >= 0, 1 <= capacity <= %d, 1 <= n_min <= n_max <= %d (got %d, %d, %d, %d)",
                    kMaxPoolCapacity, AASD_MAX_KEY, B, capacity, n_min, n_max);
    if (tok_stride < 1 || tok_stride > 0x7fffffffLL) return fail(AASD_ERR_INVALID_ARG, "pool_retrieve: tok_stride = %lld out of range", (long long)tok_stride);
    if (k < 1 || k > AASD_MAX_DRAFT) return fail(AASD_ERR_INVALID_ARG, "pool_retrieve: k = %d outside [1,%d]", k, AASD_MAX_DRAFT);
    if (C < 1 || C > AASD_MAX_CANDIDATES) return fail(AASD_ERR_INVALID_ARG, "pool_retrieve: C = %d outside [1,%d]", C, AASD_MAX_CANDIDATES);
    const bool have_table = extras != nullptr || n_extras != nullptr;
    if (have_table && (!extras || !n_extras || m < 1 || m > AASD_MAX_EXTRAS || extras_stride < 0))
        return fail(AASD_ERR_INVALID_ARG, "pool_retrieve: an extras table needs extras, n_extras, 1 <= m <= %d and extras_stride >= 0", AASD_MAX_EXTRAS);
    if (draft_extras && !have_table) return fail(AASD_ERR_INVALID_ARG, "pool_retrieve: draft_extras wanted but no extras table given");
    if (B == 0) return AASD_OK;
    if (!tokens || !len || !prompt_len || !drafts || !draft_len || !src_pos || !n_cand || !key_len || !strict)
        return fail(AASD_ERR_INVALID_ARG, "pool_retrieve: null required pointer");
    if (!pool || pool_bytes < need)
        return fail(AASD_ERR_WORKSPACE, "pool_retrieve: pool of %zu bytes needed, %zu given", need, pool ? pool_bytes : (size_t)0);
    if (((uintptr_t)pool % 16) != 0) return fail(AASD_ERR_WORKSPACE, "pool_retrieve: pool is not 16-byte aligned");
    aasd::PoolRetrieveParams q{};
    q.pool = (const char*)pool; q.lay = lay;
    aasd::RetrieveParams& p = q.r;
    p.tokens = tokens; p.tok_stride = tok_stride; p.len = len; p.prompt_len = prompt_len;
    p.B = B; p.n_min = n_min; p.n_max = n_max; p.k = k; p.C = C;
    p.extras = extras; p.n_extras = n_extras; p.m_x = have_table ? m : 0; p.extras_stride = extras_stride;
    p.drafts = drafts; p.draft_len = draft_len; p.src_pos = src_pos; p.n_cand = n_cand; p.key_len = key_len;
    p.draft_extras = draft_extras; p.strict = strict;
    if (update_first)
        hipLaunchKernelGGL(aasd::pool_step_kernel, dim3((unsigned)B), dim3((n_max - n_min + 1) * aasd::kWave), 0, (hipStream_t)stream, q);
    else
        hipLaunchKernelGGL(aasd::pool_retrieve_kernel, dim3((unsigned)B), dim3(aasd::kWave), 0, (hipStream_t)stream, q);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "pool_retrieve launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

int aasd_pool_retrieve(const void* pool, size_t pool_bytes, int32_t B, int32_t capacity, int32_t n_min, int32_t n_max,
                       const int32_t* tokens, int64_t tok_stride, const int32_t* len, const int32_t* prompt_len,
                       int32_t k, int32_t C, const int32_t* extras, const uint8_t* n_extras, int32_t m,
                       int64_t extras_stride, int32_t* drafts, int32_t* draft_len, int32_t* src_pos,
                       int32_t* n_cand, int32_t* key_len, int32_t* draft_extras, uint8_t* strict, void* stream)
{
    return pool_lookup(false, pool, pool_bytes, B, capacity, n_min, n_max, tokens, tok_stride, len, prompt_len, k, C,
                       extras, n_extras, m, extras_stride, drafts, draft_len, src_pos, n_cand, key_len, draft_extras,
                       strict, stream);
}

int aasd_pool_step(void* pool, size_t pool_bytes, int32_t B, int32_t capacity, int32_t n_min, int32_t n_max,
                   const int32_t* tokens, int64_t tok_stride, const int32_t* len, const int32_t* prompt_len,
                   int32_t k, int32_t C, const int32_t* extras, const uint8_t* n_extras, int32_t m,
                   int64_t extras_stride, int32_t* drafts, int32_t* draft_len, int32_t* src_pos,
                   int32_t* n_cand, int32_t* key_len, int32_t* draft_extras, uint8_t* strict, void* stream)
{
    return pool_lookup(true, pool, pool_bytes, B, capacity, n_min, n_max, tokens, tok_stride, len, prompt_len, k, C,
                       extras, n_extras, m, extras_stride, drafts, draft_len, src_pos, n_cand, key_len, draft_extras,
                       strict, stream);
}

size_t aasd_verify_topk_workspace_bytes(int32_t B, int32_t C, int32_t k, int32_t V, int32_t dt)
{
    if (B < 0 || C < 1 || C > AASD_MAX_CANDIDATES || k < 1 || k > AASD_MAX_DRAFT || V <= 0 || !valid_dtype(dt)) return 0;
    const int64_t rows = (int64_t)B * (1 + C * k);
    const SweepPlan pl = plan_sweep(true, rows, V, dt);
    // per-wave partials and candidate lists of the alignment-style sweep, then the K-th largest logit and the greedy pick of every row
    return align16((size_t)rows * pl.npart * (sizeof(aasd::WavePartial) + aasd::kListCap * sizeof(int32_t))) +
           (size_t)rows * (sizeof(float) + sizeof(int32_t));
}

int aasd_verify_topk(const void* logits, int32_t dt, int32_t B, int32_t C, int32_t k, int32_t V,
                     int64_t row_stride, int64_t seq_stride, const int32_t* drafts,
                     const int32_t* draft_len, int32_t topk, int32_t* accept_len, int32_t* best_cand,
                     int32_t* next_token, int32_t* row_argmax, uint8_t* tok_pass, void* workspace,
                     size_t workspace_bytes, void* stream)
{
    if (!valid_dtype(dt)) return fail(AASD_ERR_INVALID_ARG, "verify_topk: unknown dtype %d", dt);
    if (B < 0) return fail(AASD_ERR_INVALID_ARG, "verify_topk: B = %d < 0", B);
    if (C < 1 || C > AASD_MAX_CANDIDATES) return fail(AASD_ERR_INVALID_ARG, "verify_topk: C = %d outside [1,%d]", C, AASD_MAX_CANDIDATES);
    if (k < 1 || k > AASD_MAX_DRAFT) return fail(AASD_ERR_INVALID_ARG, "verify_topk: k = %d outside [1,%d]", k, AASD_MAX_DRAFT);
    if (V <= 0) return fail(AASD_ERR_INVALID_ARG, "verify_topk: V = %d <= 0", V);
    if (topk < 1 || topk > AASD_MAX_CANDSET)
        return fail(AASD_ERR_INVALID_ARG, "verify_topk: topk = %d outside [1,%d]", topk, AASD_MAX_CANDSET);
    const int32_t R = 1 + C * k;
    if (row_stride < V) return fail(AASD_ERR_INVALID_ARG, "verify_topk: row_stride %lld < V %d", (long long)row_stride, V);
    if (seq_stride < (int64_t)R * row_stride)
        return fail(AASD_ERR_INVALID_ARG, "verify_topk: seq_stride %lld < R*row_stride %lld", (long long)seq_stride, (long long)((int64_t)R * row_stride));
    if (B == 0) return AASD_OK;
    if (!logits || !drafts || !draft_len || !accept_len || !best_cand || !next_token)
        return fail(AASD_ERR_INVALID_ARG, "verify_topk: null required pointer");
    if (((uintptr_t)logits % elt_size(dt)) != 0)
        return fail(AASD_ERR_UNSUPPORTED, "verify_topk: logits pointer is not aligned to its element size");
    const size_t need = aasd_verify_topk_workspace_bytes(B, C, k, V, dt);
    if (!workspace || workspace_bytes < need)
        return fail(AASD_ERR_WORKSPACE, "verify_topk: workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
    if (((uintptr_t)workspace % 16) != 0) return fail(AASD_ERR_WORKSPACE, "verify_topk: workspace is not 16-byte aligned");

    hipStream_t s = (hipStream_t)stream;
    const int64_t rows = (int64_t)B * R;
    const SweepPlan pl = plan_sweep(true, rows, V, dt);
    aasd::WavePartial* partials = (aasd::WavePartial*)workspace;
    int32_t* lists = (int32_t*)((char*)workspace + (size_t)rows * pl.npart * sizeof(aasd::WavePartial));
    char* after = (char*)workspace + align16((size_t)rows * pl.npart * (sizeof(aasd::WavePartial) + aasd::kListCap * sizeof(int32_t)));
    float* kth = (float*)after;
    int32_t* am = (int32_t*)(after + (size_t)rows * sizeof(float));

    aasd::SweepParams sp{};
    sp.logits = logits; sp.V = V; sp.row_stride = row_stride; sp.seq_stride = seq_stride; sp.rows_per_seq = R;
    sp.next_tok = nullptr; sp.want_cand = 1; sp.cand_all = 1; sp.c = topk;
    sp.nseg = pl.nseg; sp.nseg_magic = div_magic(pl.nseg); sp.seg_vecs = pl.seg_vecs; sp.partials = partials; sp.lists = lists;
    size_t dyn = 0;
    {
        const size_t per_lane = (size_t)(pl.seg_vecs / pl.block) * elt_size(dt);
        size_t stride = (per_lane + 15) / 16 * 16;
        if ((stride / 16) % 2 == 0) stride += 16;
        if (stride * pl.block <= kMaxChunkMaxLds) { dyn = stride * pl.block; sp.cm_enabled = 1; sp.cm_stride = (int32_t)stride; }
    }
    int rc = dt == AASD_BF16 ? launch_sweep<AASD_BF16, true, false>(sp, pl, rows, dyn, s)
                             : launch_sweep<AASD_F32, true, false>(sp, pl, rows, dyn, s);
    if (rc != AASD_OK) return rc;

    aasd::RowKthParams kp{};
    kp.f.logits = logits; kp.f.V = V; kp.f.row_stride = row_stride; kp.f.rows = rows; kp.f.c = topk;
    kp.f.partials = partials; kp.f.lists = lists; kp.f.npart = pl.npart;
    kp.rows_per_seq = R; kp.seq_stride = seq_stride; kp.kth = kth; kp.argmax = am;
    const int rows_per_block = aasd::kFinishBlock / aasd::kWave;
    if (rows > kMaxUnitsPerLaunch * rows_per_block) return fail(AASD_ERR_UNSUPPORTED, "verify_topk: too many rows for one launch");
    const unsigned grid = (unsigned)((rows + rows_per_block - 1) / rows_per_block);
    if (dt == AASD_BF16) hipLaunchKernelGGL(aasd::row_kth_kernel<AASD_BF16>, dim3(grid), dim3(aasd::kFinishBlock), 0, s, kp);
    else hipLaunchKernelGGL(aasd::row_kth_kernel<AASD_F32>, dim3(grid), dim3(aasd::kFinishBlock), 0, s, kp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "row_kth launch failed: %s", hipGetErrorString(e));

    aasd::VerifyTopkTailParams tp{};
    tp.logits = logits; tp.B = B; tp.C = C; tp.k = k; tp.V = V; tp.row_stride = row_stride; tp.seq_stride = seq_stride;
    tp.drafts = drafts; tp.draft_len = draft_len; tp.kth = kth; tp.argmax = am;
    tp.accept_len = accept_len; tp.best_cand = best_cand; tp.next_token = next_token;
    tp.row_argmax = row_argmax; tp.tok_pass = tok_pass;
    if (dt == AASD_BF16) hipLaunchKernelGGL(aasd::verify_topk_tail_kernel<AASD_BF16>, dim3((unsigned)B), dim3(aasd::kWave), 0, s, tp);
    else hipLaunchKernelGGL(aasd::verify_topk_tail_kernel<AASD_F32>, dim3((unsigned)B), dim3(aasd::kWave), 0, s, tp);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "verify_topk tail launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

int aasd_build_tree(const int32_t* drafts, const int32_t* draft_len, const uint8_t* strict,
                    const int32_t* draft_extras, int32_t m, const int32_t* root_tok, int32_t B,
                    int32_t C, int32_t k, int32_t max_nodes, int32_t* node_token,
                    int32_t* node_parent, int32_t* node_depth, uint8_t* node_strict,
                    int32_t* n_nodes, uint32_t* mask, int32_t* cand_node, void* stream)
{
    if (B < 0) return fail(AASD_ERR_INVALID_ARG, "build_tree: B = %d < 0", B);
    if (k < 1 || k > AASD_MAX_DRAFT) return fail(AASD_ERR_INVALID_ARG, "build_tree: k = %d outside [1,%d]", k, AASD_MAX_DRAFT);
    if (C < 1 || C > AASD_MAX_CANDIDATES) return fail(AASD_ERR_INVALID_ARG, "build_tree: C = %d outside [1,%d]", C, AASD_MAX_CANDIDATES);
    if (m < 0 || m > AASD_MAX_EXTRAS) return fail(AASD_ERR_INVALID_ARG, "build_tree: m = %d outside [0,%d]", m, AASD_MAX_EXTRAS);
    if (draft_extras && m < 1) return fail(AASD_ERR_INVALID_ARG, "build_tree: draft_extras given with m = %d", m);
    if (max_nodes < 1 || max_nodes > AASD_MAX_TREE_NODES)
        return fail(AASD_ERR_INVALID_ARG, "build_tree: max_nodes = %d outside [1,%d]", max_nodes, AASD_MAX_TREE_NODES);
    if (B == 0) return AASD_OK;
    if (!drafts || !draft_len || !node_token || !node_parent || !node_depth || !node_strict || !n_nodes)
        return fail(AASD_ERR_INVALID_ARG, "build_tree: null required pointer");
    aasd::BuildTreeParams p{};
    p.drafts = drafts; p.draft_len = draft_len; p.strict = strict; p.draft_extras = draft_extras; p.m_x = m;
    p.root_tok = root_tok; p.B = B; p.C = C; p.k = k; p.max_nodes = max_nodes;
    p.w_magic = div_magic((max_nodes + 31) / 32);
    p.node_token = node_token; p.node_parent = node_parent; p.node_depth = node_depth; p.node_strict = node_strict;
    p.n_nodes = n_nodes; p.mask = mask; p.cand_node = cand_node;
    hipLaunchKernelGGL(aasd::build_tree_kernel, dim3((unsigned)B), dim3(aasd::kTreeBlock), 0, (hipStream_t)stream, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "build_tree launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

size_t aasd_verify_tree_workspace_bytes(int32_t B, int32_t N, int32_t V, int32_t dt)
{
    if (B < 0 || N < 1 || N > AASD_MAX_TREE_NODES || V <= 0 || !valid_dtype(dt)) return 0;
    const int64_t rows = (int64_t)B * N;
    const SweepPlan pl = plan_tree_sweep(rows, V, dt);
    return (size_t)rows * pl.npart * sizeof(aasd::WavePartial);
}

int aasd_verify_tree(const void* logits, int32_t dt, int32_t B, int32_t N, int32_t V,
                     int64_t row_stride, int64_t seq_stride, const int32_t* node_token,
                     const int32_t* node_parent, const uint8_t* node_strict,
                     const int32_t* n_nodes, float alpha, float beta, uint32_t flags,
                     int32_t* accept_len, int32_t* best_node, int32_t* accept_path,
                     int32_t* next_token, float* row_entropy, float* row_pmax,
                     int32_t* row_argmax, float* node_p, float* node_delta,
                     uint32_t* near_count, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!valid_dtype(dt)) return fail(AASD_ERR_INVALID_ARG, "verify_tree: unknown dtype %d", dt);
    if (B < 0) return fail(AASD_ERR_INVALID_ARG, "verify_tree: B = %d < 0", B);
    if (N < 1 || N > AASD_MAX_TREE_NODES) return fail(AASD_ERR_INVALID_ARG, "verify_tree: N = %d outside [1,%d]", N, AASD_MAX_TREE_NODES);
    if (V <= 0) return fail(AASD_ERR_INVALID_ARG, "verify_tree: V = %d <= 0", V);
    if (row_stride < V) return fail(AASD_ERR_INVALID_ARG, "verify_tree: row_stride %lld < V %d", (long long)row_stride, V);
    if (seq_stride < (int64_t)N * row_stride)
        return fail(AASD_ERR_INVALID_ARG, "verify_tree: seq_stride %lld < N*row_stride %lld", (long long)seq_stride, (long long)((int64_t)N * row_stride));
    if (flags & ~AASD_VERIFY_NO_CLAMP) return fail(AASD_ERR_INVALID_ARG, "verify_tree: unknown flag bits 0x%x", flags);
    if (B == 0) return AASD_OK;
    if (!logits || !node_token || !node_parent || !n_nodes || !accept_len || !best_node || !next_token)
        return fail(AASD_ERR_INVALID_ARG, "verify_tree: null required pointer");
    if (((uintptr_t)logits % elt_size(dt)) != 0)
        return fail(AASD_ERR_UNSUPPORTED, "verify_tree: logits pointer is not aligned to its element size");
    const size_t need = aasd_verify_tree_workspace_bytes(B, N, V, dt);
    if (!workspace || workspace_bytes < need)
        return fail(AASD_ERR_WORKSPACE, "verify_tree: workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
    if (((uintptr_t)workspace % 16) != 0) return fail(AASD_ERR_WORKSPACE, "verify_tree: workspace is not 16-byte aligned");

    hipStream_t s = (hipStream_t)stream;
    const int64_t rows = (int64_t)B * N;
    const SweepPlan pl = plan_tree_sweep(rows, V, dt);
    aasd::SweepParams sp{};
    sp.logits = logits; sp.V = V; sp.row_stride = row_stride; sp.seq_stride = seq_stride; sp.rows_per_seq = N;
    sp.rows_used = n_nodes;
    sp.c = 1; sp.nseg = pl.nseg; sp.nseg_magic = div_magic(pl.nseg); sp.seg_vecs = pl.seg_vecs; sp.partials = (aasd::WavePartial*)workspace;
    int rc = dt == AASD_BF16 ? launch_sweep_used<AASD_BF16>(sp, pl, B, s) : launch_sweep_used<AASD_F32>(sp, pl, B, s);
    if (rc != AASD_OK) return rc;

    aasd::VerifyTreeParams tp{};
    tp.logits = logits; tp.B = B; tp.N = N; tp.V = V; tp.row_stride = row_stride; tp.seq_stride = seq_stride;
    tp.node_token = node_token; tp.node_parent = node_parent; tp.node_strict = node_strict; tp.n_nodes = n_nodes;
    tp.alpha = alpha; tp.beta = beta; tp.flags = flags;
    tp.accept_len = accept_len; tp.best_node = best_node; tp.accept_path = accept_path; tp.next_token = next_token;
    tp.node_p = node_p; tp.node_delta = node_delta; tp.near_count = near_count;
    tp.row_entropy = row_entropy; tp.row_pmax = row_pmax; tp.row_argmax = row_argmax;
    tp.partials = (const aasd::WavePartial*)workspace; tp.npart = pl.npart;
    if (dt == AASD_BF16)
        hipLaunchKernelGGL(aasd::verify_tree_kernel<AASD_BF16>, dim3((unsigned)B), dim3(aasd::kVerifyTreeBlock), 0, s, tp);
    else
        hipLaunchKernelGGL(aasd::verify_tree_kernel<AASD_F32>, dim3((unsigned)B), dim3(aasd::kVerifyTreeBlock), 0, s, tp);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "verify_tree launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

}  // extern "C"
