// SOAR NVFP4 weight quantization for MI355X (gfx950): HIP kernels and C-ABI.
//
// Path (arXiv 2605.12245, Algorithm 1 with T = 1 and beta = 1), three streaming
// kernels per group of tensors:
//   absmax   max|W|                                     -> alpha0       (Eq. 1)
//   stats    per block: Delta0, Q0, a = sum w q, b = sum q^2            (Eq. 1-2)
//            tensor:    N = sum a Delta0, M = sum b Delta0^2 -> alpha1  (Eq. 5)
//   search   per block: Delta* = (a/b)/alpha1 (Eq. 6), centre = E4M3(Delta*)
//            (Appendix D), Q1 = Q_FP4(W/(alpha1 Delta*)), search of the stored
//            scale over centre-K..centre+K by Eq. 8, pack, error sum
//
// Algorithm 1 in full (T iterations, a grid of factors beta for the quantization
// scale, early stop) runs as absmax, one pass that builds the Eq. 1-2 state, and
// one arithmetic-bound pass per iteration; see k_iter.
//
// Work decomposition: one lane owns one 16-element block (two 128-bit loads for
// bf16), so every per-block reduction is a register chain with no cross-lane
// traffic.  A workgroup of 256 lanes owns "tiles" of 256 consecutive blocks.
// The two tensor-wide sums are binary64 adjacent-pair trees over the flat block
// index: LDS staging of a few tiles, a DPP wave tree, a 4-wave step and a
// binary-counter stack reproduce that tree exactly for any power-of-two number
// of tiles per workgroup.  One launch serves up to kGroupMax tensors (each with
// its own range of workgroups) so that small tensors do not pay a launch each.
//
// Tensor-wide results are finished by the last workgroup of a tensor to arrive
// (two-level arrival counters, no spinning, no cache-wide fences).
//
// Build: hipcc --offload-arch=gfx950 -O3 -ffp-contract=off (no fast-math): every
// float operation below is a separate IEEE binary32 operation unless written as
// __builtin_fmaf, divisions are correctly rounded, subnormals are kept.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <atomic>
#include <chrono>
#include <cstring>
#include <mutex>
#include <vector>

#include "soar.h"
#include "soar_device.hpp"
#include "soar_single_step.hpp"
#include "soar_iterated.hpp"
#include "soar_mxfp4.hpp"
#include "soar_stored_form.hpp"

// Workspace of soar_quantize_static: the control slots of one launch and one float per block for a
// tensor of at most kStaticMaxBlocks blocks.  One copy per GPU, held until the process ends; in host
// code the name below is only a handle for hipGetSymbolAddress, never an address.
constexpr int64_t kStaticMaxBlocks = (int64_t)1 << 22;        // 2^26 weights, e.g. 8192 x 8192
constexpr size_t kStaticScratchBytes = (size_t)kGroupMax * kSlotBytes + (size_t)kStaticMaxBlocks * sizeof(float);
static_assert(kStaticMaxBlocks == SOAR_STATIC_MAX_BLOCKS, "limit stated in soar.h");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Diagnostic counters of the certified search (count_search), one set per GPU.
static __device__ unsigned long long search_stats_words[4];

namespace {

// ------------------------------------------------------------------ host side
constexpr int kMaxDevices = 64;

std::atomic<bool> g_search_stats{false};

// device address of the diagnostic counters on the current device, or null while they are off
unsigned long long *search_stats_address()
{
    if (!g_search_stats.load(std::memory_order_relaxed)) return nullptr;
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(search_stats_words)) != hipSuccess) return nullptr;
    return static_cast<unsigned long long *>(p);
}

// device address of `scratch` on the current device, looked up once per device; null on failure
void *static_scratch_address()
{
    static std::once_flag once[kMaxDevices];
    static void *address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::call_once(once[dev], [dev] {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) == hipSuccess) address[dev] = p;
    });
    return address[dev];
}

// what the one-launch kernel needs to know of the current device, looked up once per device
struct DeviceFacts {
    int compute_units = 0;            // 0: not known, the one-launch kernel is not used
    int wall_clock_khz = 100000;
};
const DeviceFacts &device_facts()
{
    static std::once_flag once[kMaxDevices];
    static DeviceFacts facts[kMaxDevices];
    static const DeviceFacts none;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return none;
    std::call_once(once[dev], [dev] {
        int cu = 0, khz = 0;
        if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cu > 0)
            facts[dev].compute_units = cu;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0)
            facts[dev].wall_clock_khz = khz;
    });
    return facts[dev];
}

// a new 64-bit value for every call: half of the token of a one-launch kernel
uint64_t next_nonce()
{
    static std::atomic<uint64_t> state{(uint64_t)std::chrono::steady_clock::now().time_since_epoch().count() * kResOdd};
    return state.fetch_add(0xD1B54A32D192ED03ull, std::memory_order_relaxed);
}

// Launch shape of the one-launch kernel for a tensor of nblk blocks on a GPU of `cu` compute units: at most
// one workgroup per compute unit (and kResMaxWG), so that the whole grid can be on the machine at once.
struct ResidentPlan { int L, R; uint32_t G; };
bool resident_plan(int64_t nblk, int cu, ResidentPlan &plan)
{
    const int64_t wgs = cu < kResMaxWG ? cu : kResMaxWG;
    if (wgs < 1) return false;
    int L = 256, R = 1;
    if (nblk > 256 * wgs) {
        L = 1024;
        while (R <= kResMaxPer && nblk > (int64_t)L * R * wgs) R <<= 1;
        if (R > kResMaxPer) return false;
    }
    plan.L = L;
    plan.R = R;
    plan.G = (uint32_t)((nblk + (int64_t)L * R - 1) / ((int64_t)L * R));
    return true;
}

// Two one-launch kernels that start at the same time on two streams can each take part of the compute
// units and then wait for the rest in vain (until the bounded wait gives up).  Calls on one stream are
// ordered by the stream.  For calls that arrive on a different stream than the one-launch kernel before
// them, this asks whether that earlier stream has drained; if it has not (or the question cannot be asked:
// either stream is being captured into a graph), the caller takes the three-pass path for this call.
// Best effort: replays of captured graphs and other processes on the same GPU are not seen here; the
// bounded wait and SOAR_STATUS_GAVE_UP cover those.
bool resident_may_start(hipStream_t st)
{
    static std::mutex mu[kMaxDevices];
    static hipStream_t last[kMaxDevices] = {};
    static bool have_last[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) return false;
    if (cap != hipStreamCaptureStatusNone) return true;      // recorded, not started: nothing to track
    std::lock_guard<std::mutex> lock(mu[dev]);
    if (have_last[dev] && last[dev] != st) {
        hipStreamCaptureStatus cap_last = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(last[dev], &cap_last) == hipSuccess) {
            if (cap_last != hipStreamCaptureStatusNone) return false;     // a query would break that capture
            const hipError_t q = hipStreamQuery(last[dev]);
            if (q == hipErrorNotReady) return false;          // may still be running: do not start beside it
            if (q != hipSuccess) (void)hipGetLastError();
        } else {
            (void)hipGetLastError();                          // a stream that no longer exists has nothing in flight
        }
    }
    last[dev] = st;
    have_last[dev] = true;
    return true;
}

template <int DT, int METHOD>
void launch_resident(const ResidentPlan &plan, const Task &t, const ResidentArgs &a, hipStream_t st)
{
    const dim3 grid(plan.G);
    if (plan.L == 256) hipLaunchKernelGGL((k_resident<DT, METHOD, 256, 1>), grid, dim3(256), 0, st, t, a);
    else if (plan.R == 1) hipLaunchKernelGGL((k_resident<DT, METHOD, 1024, 1>), grid, dim3(1024), 0, st, t, a);
    else if (plan.R == 2) hipLaunchKernelGGL((k_resident<DT, METHOD, 1024, 2>), grid, dim3(1024), 0, st, t, a);
    else hipLaunchKernelGGL((k_resident<DT, METHOD, 1024, 4>), grid, dim3(1024), 0, st, t, a);
}

thread_local bool t_no_event_timing = false;      // set while an entry point that must not create events runs

struct Timing {
    bool enabled = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev[SOAR_KERNEL_COUNT];
};
Timing g_timing;

struct ScopedTimer {
    int id;
    hipStream_t st;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ScopedTimer(int id_, hipStream_t st_) : id(id_), st(st_)
    {
        if (!g_timing.enabled || t_no_event_timing) return;
        // timing only: no system-scope fence (cache write-back and invalidation) with the record, which would be
        // charged to the kernel between the two events and to the one after
        if (hipEventCreateWithFlags(&e0, hipEventDisableSystemFence) != hipSuccess ||
            hipEventCreateWithFlags(&e1, hipEventDisableSystemFence) != hipSuccess) { e0 = e1 = nullptr; return; }
        (void)hipEventRecord(e0, st);
    }
    ~ScopedTimer()
    {
        if (!e0) return;
        (void)hipEventRecord(e1, st);
        g_timing.ev[id].emplace_back(e0, e1);
    }
};

bool valid_params(const soar_params *p)
{
    if (!p || p->struct_size != sizeof(soar_params)) return false;
    if (p->method < SOAR_METHOD_RTN || p->method > SOAR_METHOD_DSS_ONLY) return false;
    if (p->block != 16) return false;
    if (p->iters < 1 || p->iters > kMaxIters || p->n_beta < 1 || p->n_beta > kMaxBeta) return false;
    if (!(p->beta_lo > 0.0f) || !(p->beta_hi >= p->beta_lo) || !(p->beta_hi < 1e30f)) return false;
    if (!(p->early_stop_rel >= 0.0f) || !(p->early_stop_rel < 1e30f)) return false;
    if (p->dd_mode != SOAR_DD_WINDOW && p->dd_mode != SOAR_DD_BRACKET) return false;
    if (p->method == SOAR_METHOD_RTN &&
        (p->iters != 1 || p->n_beta != 1 || p->beta_lo != 1.0f || p->dd_mode != SOAR_DD_WINDOW))
        return false;
    if (p->method == SOAR_METHOD_CJSO_ONLY &&
        (p->n_beta != 1 || p->beta_lo != 1.0f || p->dd_mode != SOAR_DD_WINDOW || p->dss_radius != 0))
        return false;
    if (p->method == SOAR_METHOD_DSS_ONLY && p->dd_mode != SOAR_DD_WINDOW) return false;
    if (p->dss_radius < 0 || p->dss_radius > 125) return false;
    if (p->search_mode != SOAR_SEARCH_AUTO && p->search_mode != SOAR_SEARCH_FULL) return false;
    if (p->tiles_per_wg < 0 || p->tiles_per_wg > 65536 || (p->tiles_per_wg & (p->tiles_per_wg - 1))) return false;
    // the maximum and the search deal their tiles round-robin: any count will do
    if (p->tiles_per_wg_absmax < 0 || p->tiles_per_wg_absmax > 65536 || p->tiles_per_wg_search < 0 || p->tiles_per_wg_search > 65536)
        return false;
    if (p->streams < 0 || p->streams > kLanes) return false;
    if (p->resident != SOAR_RESIDENT_AUTO && p->resident != SOAR_RESIDENT_NEVER) return false;
    if (p->resident_wait_us < 0) return false;
    return true;
}

soar_status check_shape(int64_t rows, int64_t cols, int64_t ld)
{
    if (rows <= 0 || cols <= 0 || cols % 16 != 0 || ld < cols) return SOAR_ERR_SHAPE;
    // block count must fit the kernels' 32-bit block index with a few tiles of slack
    if (rows > (int64_t)1 << 31 || cols > (int64_t)1 << 31) return SOAR_ERR_SHAPE;
    if (rows * (cols / 16) > ((int64_t)1 << 31) - 16 * kWG) return SOAR_ERR_SHAPE;
    return SOAR_OK;
}

soar_status check_matrix_ptr(const void *p, int dtype, int64_t ld)
{
    const int64_t es = dtype == SOAR_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return SOAR_ERR_ALIGN;
    if ((ld * es) % 16 != 0) return SOAR_ERR_ALIGN;
    return SOAR_OK;
}

// Algorithm 1 beyond the single-step settings
bool iterated_params(const soar_params *p)
{
    return p->method == SOAR_METHOD_CJSO_ONLY || p->method == SOAR_METHOD_DSS_ONLY || p->iters != 1 || p->n_beta != 1 || p->beta_lo != 1.0f || p->dd_mode != SOAR_DD_WINDOW;
}

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

// bytes of per-block workspace (one float) of one tensor
size_t per_block_bytes(int64_t rows, int64_t cols)
{
    const size_t nblk = (size_t)(rows * (cols / 16));
    return align256(nblk * sizeof(float));
}

// Tiles per workgroup the three passes of the single-step path ask for.  A call of one launch group runs its
// kernels one after the other, and four tiles suit each of them best.  A call of several groups has kernels of
// two groups on the machine at once (see SecondLane), and how their workgroups share the compute units decides
// the step: with 8 tiles per workgroup in the statistics pass and 16 in the search the full-model workload
// takes 7.26 ms instead of 8.08 (swept over 1..4 x 4..32 x 8..32: profiles/config4_launch_shape_sweep.md),
// although the search alone is 5 % slower that way; plain NVFP4 (two passes) likes 8 in its search.
struct WantedShapes { uint32_t absmax, stats, search; };
WantedShapes wanted_shapes(bool several_groups, int method, bool iterated, bool one_pass, int64_t bytes)
{
    if (!several_groups || iterated || one_pass) return {(uint32_t)kStage, (uint32_t)kStage, (uint32_t)kStage};
    // a tensor that is a launch group by itself and larger than the last-level cache streams from HBM in every
    // pass; plain NVFP4 has two passes only
    if (method == SOAR_METHOD_RTN || bytes > kGroupByteCap) return {(uint32_t)kStage, (uint32_t)kStage, 8u};
    return {(uint32_t)kStage, 8u, 16u};
}

// tiles per workgroup of an arithmetic-bound searching kernel over a launch of `tiles` tiles
constexpr int64_t kSearchMinWg = 2048;
uint32_t search_tiles_per_wg(int64_t tiles)
{
    uint32_t tpw = 16;
    while (tpw > 1 && tiles / tpw < kSearchMinWg) tpw >>= 1;
    return tpw;
}

// addressing and launch shapes of one tensor; the workspace fields and the first workgroups stay unset
Task make_task(const void *w, int64_t rows, int64_t cols, int64_t ld, const WantedShapes &forced, const WantedShapes &want)
{
    Task t;
    std::memset(&t, 0, sizeof(t));
    t.w = w;
    t.ld = ld;
    t.bpr = (uint32_t)(cols / 16);
    t.nblk = (uint32_t)(rows * (cols / 16));
    t.contiguous = (ld == cols) ? 1u : 0u;
    const uint32_t tiles = (t.nblk + kWG - 1) / kWG;
    auto shape = [&](uint32_t wanted, uint32_t forced_tpw) {
        Shape sh;
        uint32_t tpw = 1;
        while (tpw < wanted && tpw * 2 <= tiles) tpw <<= 1;
        if (forced_tpw) tpw = forced_tpw;
        while ((tiles + tpw - 1) / tpw > (uint32_t)kMaxPartials) tpw <<= 1;
        sh.tiles_per_wg = tpw;
        sh.n_wg = (tiles + tpw - 1) / tpw;
        sh.wg_begin = 0;
        return sh;
    };
    const Shape base = shape(want.stats, forced.stats);
    t.tiles_per_wg = base.tiles_per_wg;
    t.n_wg = base.n_wg;
    t.absmax = shape(want.absmax, forced.absmax);
    t.search = shape(want.search, forced.search);
    return t;
}

#define SOAR_LAUNCH_CHECK()                                  \
    do {                                                     \
        if (hipGetLastError() != hipSuccess) return SOAR_ERR_HIP; \
    } while (0)

soar_status validate_tensor(const soar_tensor_desc &d, const soar_params *params)
{
    if (!d.d_w || !d.d_codes || !d.d_scales || !d.d_global_scale) return SOAR_ERR_NULL;
    if (d.dtype != SOAR_BF16 && d.dtype != SOAR_FP32) return SOAR_ERR_DTYPE;
    if (!valid_params(params)) return SOAR_ERR_PARAM;
    soar_status s = check_shape(d.rows, d.cols, d.ld_elems);
    if (s != SOAR_OK) return s;
    s = check_matrix_ptr(d.d_w, d.dtype, d.ld_elems);
    if (s != SOAR_OK) return s;
    if (reinterpret_cast<uintptr_t>(d.d_codes) % 8 != 0) return SOAR_ERR_ALIGN;
    return SOAR_OK;
}

// how many tensors starting at `first` go into one launch
int64_t weight_bytes(const soar_tensor_desc &d) { return d.rows * d.cols * (d.dtype == SOAR_BF16 ? 2 : 4); }

constexpr int64_t kOnePassByteCap = (int64_t)1 << 29;    // larger launches gain nothing more (measured: 2^29 .. 2^31)

// bytes of weights one launch may cover (beyond its first tensor)
int64_t group_byte_cap(const soar_tensor_desc *descs, const soar_params *params)
{
    // with the maximum supplied there is one pass only: nothing to keep in the last-level cache
    if (descs[0].d_amax_in) return kOnePassByteCap;
    (void)params;
    return kGroupByteCap;      // a group stays in the 256 MiB last-level cache from pass to pass, iteration to iteration
}

int32_t group_end(int32_t n, const soar_tensor_desc *descs, int32_t first, int64_t cap)
{
    int64_t bytes = weight_bytes(descs[first]);
    int32_t j = first + 1;
    while (j < n && j - first < kGroupMax && descs[j].dtype == descs[first].dtype &&
           bytes + weight_bytes(descs[j]) <= cap) {
        bytes += weight_bytes(descs[j]);
        ++j;
    }
    return j;
}

// most per-block workspace any one launch of the batch needs
size_t max_group_per_block_bytes(int32_t n, const soar_tensor_desc *descs, int64_t cap, int32_t *n_groups)
{
    size_t most = 0;
    int32_t groups = 0;
    for (int32_t i = 0; i < n;) {
        const int32_t j = group_end(n, descs, i, cap);
        size_t sum = 0;
        for (int32_t k = i; k < j; ++k) sum += per_block_bytes(descs[k].rows, descs[k].cols);
        if (sum > most) most = sum;
        i = j;
        ++groups;
    }
    if (n_groups) *n_groups = groups;
    return most;
}

// A batch of two or more launch groups is spread over two streams (the caller's
// and one of the library's own, forked and joined with events), so that the
// memory-only and the arithmetic-heavy kernels of different groups overlap.
// Each stream works in its own half of the workspace.

size_t lane_workspace_bytes(size_t group_per_block) { return (size_t)kGroupMax * kSlotBytes + group_per_block; }

size_t batch_workspace_bytes(int32_t n, const soar_tensor_desc *descs, const soar_params *params)
{
    int32_t groups = 0;
    const size_t most = max_group_per_block_bytes(n, descs, group_byte_cap(descs, params), &groups);
    return (groups > 1 ? kLanes : 1) * lane_workspace_bytes(most);
}

// What a batch of two or more launch groups needs beside the caller's stream: one stream per GPU
// (default priority) and the two events that fork it off the caller's stream and join it back.  Created
// on the first such call on a device, under std::call_once, shared by all callers and never destroyed.
// An event is recorded and waited for under the lock, so that two host threads cannot wait for each
// other's record.
struct SecondLane {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    std::mutex mu;
    bool usable = false;

    // `from` -> `to`: work enqueued on `to` after this call starts after what `from` holds now
    bool order(hipEvent_t ev, hipStream_t from, hipStream_t to)
    {
        std::lock_guard<std::mutex> lock(mu);
        return hipEventRecord(ev, from) == hipSuccess && hipStreamWaitEvent(to, ev, 0) == hipSuccess;
    }
};

SecondLane *second_lane()
{
    static std::once_flag once[kMaxDevices];
    static SecondLane lanes[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::call_once(once[dev], [dev] {
        SecondLane &l = lanes[dev];
        l.usable = hipStreamCreateWithFlags(&l.stream, hipStreamNonBlocking) == hipSuccess &&
                   hipEventCreateWithFlags(&l.fork, hipEventDisableTiming) == hipSuccess &&
                   hipEventCreateWithFlags(&l.join, hipEventDisableTiming) == hipSuccess;
    });
    return lanes[dev].usable ? &lanes[dev] : nullptr;
}

// grids: every pass has its own number of workgroups (Task::absmax, the base shape, Task::search)
template <int DT>
soar_status launch_group(const Batch &b, uint32_t wg_absmax, uint32_t wg_stats, uint32_t wg_search, int method, hipStream_t st)
{
    if (b.t[0].amax_in == nullptr) {       // all tensors of a batch supply their maximum, or none does
        ScopedTimer t(SOAR_KERNEL_ABSMAX, st);
        hipLaunchKernelGGL(k_absmax<DT>, dim3(wg_absmax), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
    }
    if (method == SOAR_METHOD_SOAR) {
        {
            ScopedTimer t(SOAR_KERNEL_STATS, st);
            hipLaunchKernelGGL(k_stats<DT>, dim3(wg_stats), dim3(kWG), 0, st, b);
            SOAR_LAUNCH_CHECK();
        }
        ScopedTimer t(SOAR_KERNEL_SEARCH, st);
        hipLaunchKernelGGL((k_search<DT, SOAR_METHOD_SOAR>), dim3(wg_search), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
    } else {
        ScopedTimer t(SOAR_KERNEL_SEARCH, st);
        hipLaunchKernelGGL((k_search<DT, SOAR_METHOD_RTN>), dim3(wg_search), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
    }
    return SOAR_OK;
}

// dynamic LDS of k_iter (see there); the two-pass condition mirrors the kernel's
size_t iter_lds_bytes(const Batch &b)
{
    size_t bytes = ((size_t)b.n_beta * 4 + 255) / 256 * 256;
    if (b.n_beta >= 4 && b.n_beta <= kMaxListBeta && !b.full_search) bytes += (size_t)b.n_beta * kWG;
    return bytes;
}

// absmax, the Eq. 1-2 state, then one launch per iteration; a tensor that has
// stopped early (or is degenerate) makes its workgroups of the later launches return at once
template <int DT>
soar_status launch_group_iter(Batch &b, uint32_t wg_absmax, uint32_t total_wg, int iters, hipStream_t st)
{
    {
        ScopedTimer t(SOAR_KERNEL_ABSMAX, st);
        hipLaunchKernelGGL(k_absmax<DT>, dim3(wg_absmax), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
    }
    {
        ScopedTimer t(SOAR_KERNEL_ITER_INIT, st);
        hipLaunchKernelGGL(k_iter_init<DT>, dim3(total_wg), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
    }
    // one pair of timing events round all iterations of the group: launches that find their tensors stopped
    // last about a microsecond, less than what an event pair of their own would add
    ScopedTimer t(SOAR_KERNEL_ITER, st);
    for (int it = 0; it < iters; ++it) {
        b.iter_t = it;
        if (b.arm == SOAR_METHOD_CJSO_ONLY) hipLaunchKernelGGL(k_cjso<DT>, dim3(total_wg), dim3(kWG), 0, st, b);
        else hipLaunchKernelGGL(k_iter<DT>, dim3(total_wg), dim3(kWG), iter_lds_bytes(b), st, b);
        SOAR_LAUNCH_CHECK();
    }
    return SOAR_OK;
}

soar_status run_batch(int32_t n, const soar_tensor_desc *descs, const soar_params *params, void *d_workspace,
                      size_t workspace_bytes, hipStream_t st)
{
    if (n < 0) return SOAR_ERR_SHAPE;
    if (n > 0 && !descs) return SOAR_ERR_NULL;
    if (!params) return SOAR_ERR_NULL;
    if (!valid_params(params)) return SOAR_ERR_PARAM;
    for (int32_t k = 0; k < n; ++k) {
        soar_status s = validate_tensor(descs[k], params);
        if (s != SOAR_OK) return s;
    }
    bool iterated = iterated_params(params);
    for (int32_t k = 0; k < n; ++k) iterated = iterated || descs[k].d_iters_run || descs[k].d_sse_trace;
    if (iterated && params->method == SOAR_METHOD_RTN) return SOAR_ERR_PARAM;
    for (int32_t k = 0; k < n; ++k) {
        if ((descs[k].d_amax_in != nullptr) != (descs[0].d_amax_in != nullptr)) return SOAR_ERR_PARAM;
        if (descs[k].d_amax_in && params->method != SOAR_METHOD_RTN) return SOAR_ERR_PARAM;
    }

    if (n == 0) return SOAR_OK;
    if (!d_workspace || reinterpret_cast<uintptr_t>(d_workspace) % 256 != 0) return SOAR_ERR_WORKSPACE;
    if (workspace_bytes < batch_workspace_bytes(n, descs, params)) return SOAR_ERR_WORKSPACE;

    // one tensor, single-step settings, default launch shape: the whole path in one launch that keeps the
    // tensor in registers, if its grid fits the GPU (see k_resident); only the slot's flag words are used
    ResidentPlan plan;
    if (n == 1 && !iterated && !descs[0].d_amax_in && params->tiles_per_wg == 0 && params->tiles_per_wg_absmax == 0 &&
        params->tiles_per_wg_search == 0 && params->resident == SOAR_RESIDENT_AUTO &&
        resident_plan(descs[0].rows * (descs[0].cols / 16), device_facts().compute_units, plan) &&
        (plan.G == 1 || resident_may_start(st))) {
        const soar_tensor_desc &d = descs[0];
        Task t = make_task(d.d_w, d.rows, d.cols, d.ld_elems, WantedShapes{0u, 0u, 0u}, wanted_shapes(false, params->method, false, false, 0));
        t.codes = d.d_codes;
        t.scales = d.d_scales;
        t.gscale = d.d_global_scale;
        t.sse = d.d_sse;
        t.status = d.d_status;
        char *slot = static_cast<char *>(d_workspace);
        t.ctrl = reinterpret_cast<Ctrl *>(slot);
        t.part = reinterpret_cast<double *>(slot + kZeroedBytes);
        ResidentArgs a;
        a.radius = params->dss_radius;
        a.full_search = params->search_mode == SOAR_SEARCH_FULL ? 1 : 0;
        a.search_stats = search_stats_address();
        a.nonce = next_nonce();
        const uint64_t us = params->resident_wait_us > 0 ? (uint64_t)params->resident_wait_us : 2000000ull;
        a.wait_ticks = us * (uint64_t)device_facts().wall_clock_khz / 1000ull;
        const bool rtn = params->method == SOAR_METHOD_RTN;
        ScopedTimer tm(SOAR_KERNEL_RESIDENT, st);
        if (d.dtype == SOAR_BF16) {
            if (rtn) launch_resident<SOAR_BF16, SOAR_METHOD_RTN>(plan, t, a, st);
            else launch_resident<SOAR_BF16, SOAR_METHOD_SOAR>(plan, t, a, st);
        } else {
            if (rtn) launch_resident<SOAR_FP32, SOAR_METHOD_RTN>(plan, t, a, st);
            else launch_resident<SOAR_FP32, SOAR_METHOD_SOAR>(plan, t, a, st);
        }
        SOAR_LAUNCH_CHECK();
        return SOAR_OK;
    }

    int32_t n_groups = 0;
    const int64_t cap = group_byte_cap(descs, params);
    const size_t lane_bytes = lane_workspace_bytes(max_group_per_block_bytes(n, descs, cap, &n_groups));
    const int lanes = (n_groups > 1 && params->streams != 1) ? kLanes : 1;
    char *base = static_cast<char *>(d_workspace);

    hipStream_t lane_stream[kLanes] = {st, st};
    SecondLane *second = nullptr;
    if (lanes > 1) {
        second = second_lane();
        if (!second) return SOAR_ERR_HIP;
        lane_stream[1] = second->stream;
    }
    soar_status result = SOAR_OK;
    {
        ScopedTimer t(SOAR_KERNEL_INIT, st);
        for (int l = 0; l < lanes && result == SOAR_OK; ++l) {
            hipLaunchKernelGGL(k_init, dim3(kGroupMax * kInitSplit), dim3(kWG), 0, st, base + (size_t)l * lane_bytes);
            if (hipGetLastError() != hipSuccess) result = SOAR_ERR_HIP;
        }
    }
    if (lanes > 1 && result == SOAR_OK && !second->order(second->fork, st, lane_stream[1])) result = SOAR_ERR_HIP;
    int32_t g = 0;
    for (int32_t i = 0; i < n && result == SOAR_OK; ++g) {
        const int32_t j = group_end(n, descs, i, cap);
        const int lane = g % lanes;
        char *lane_base = base + (size_t)lane * lane_bytes;
        Batch b;
        std::memset(&b, 0, sizeof(b));
        b.n = (uint32_t)(j - i);
        b.radius = params->dss_radius;
        b.full_search = params->search_mode == SOAR_SEARCH_FULL ? 1 : 0;
        b.search_stats = search_stats_address();
        b.n_beta = params->n_beta;
        b.dd_mode = params->dd_mode;
        b.beta_lo = params->beta_lo;
        b.beta_hi = params->beta_hi;
        b.early_stop_rel = params->early_stop_rel;
        b.arm = params->method;
        // The searching iterated kernels are arithmetic-bound: up to 16 tiles per workgroup, as long as the launch
        // keeps kSearchMinWg workgroups (a few rounds of what the GPU holds at once) to balance over: the
        // full-model workload takes 267 ms per step that way, 299 with one tile per workgroup.  (The closed-form
        // arm has no search and streams like the single-step kernels.)
        const bool searching = iterated && params->method != SOAR_METHOD_CJSO_ONLY;
        const uint32_t tpw = (uint32_t)params->tiles_per_wg;
        uint32_t searching_tpw = 0;
        if (searching) {
            int64_t group_tiles = 0;
            for (int32_t k = i; k < j; ++k) group_tiles += (descs[k].rows * (descs[k].cols / 16) + kWG - 1) / kWG;
            searching_tpw = search_tiles_per_wg(group_tiles);
        }
        uint32_t wg = 0, wg_absmax = 0, wg_search = 0;
        char *per_block = lane_base + (size_t)kGroupMax * kSlotBytes;
        for (int32_t k = i; k < j; ++k) {
            const soar_tensor_desc &d = descs[k];
            const WantedShapes forced = {params->tiles_per_wg_absmax ? (uint32_t)params->tiles_per_wg_absmax : tpw, tpw,
                                         params->tiles_per_wg_search ? (uint32_t)params->tiles_per_wg_search : tpw};
            const WantedShapes want = searching ? WantedShapes{searching_tpw, searching_tpw, searching_tpw}
                                                : wanted_shapes(n_groups > 1, params->method, iterated, d.d_amax_in != nullptr,
                                                                weight_bytes(d));
            Task t = make_task(d.d_w, d.rows, d.cols, d.ld_elems, forced, want);
            t.iters_run = d.d_iters_run;
            t.trace = d.d_sse_trace;
            t.amax_in = d.d_amax_in;
            t.codes = d.d_codes;
            t.scales = d.d_scales;
            t.gscale = d.d_global_scale;
            t.sse = d.d_sse;
            t.status = d.d_status;
            t.wg_begin = wg;
            wg += t.n_wg;
            t.absmax.wg_begin = wg_absmax;
            wg_absmax += t.absmax.n_wg;
            t.search.wg_begin = wg_search;
            wg_search += t.search.n_wg;
            char *slot = lane_base + (size_t)(k - i) * kSlotBytes;
            t.ctrl = reinterpret_cast<Ctrl *>(slot);
            t.counters = reinterpret_cast<uint32_t *>(slot + kCtrlBytes);
            t.slot_max = reinterpret_cast<uint32_t *>(slot + kCtrlBytes + kCountersBytes);
            t.part = reinterpret_cast<double *>(slot + kZeroedBytes);
            t.rho = reinterpret_cast<float *>(per_block);
            per_block += align256((size_t)t.nblk * sizeof(float));
            b.t[k - i] = t;
        }
        if (iterated)
            result = descs[i].dtype == SOAR_BF16 ? launch_group_iter<SOAR_BF16>(b, wg_absmax, wg, params->iters, lane_stream[lane])
                                                 : launch_group_iter<SOAR_FP32>(b, wg_absmax, wg, params->iters, lane_stream[lane]);
        else
            result = descs[i].dtype == SOAR_BF16
                         ? launch_group<SOAR_BF16>(b, wg_absmax, wg, wg_search, params->method, lane_stream[lane])
                         : launch_group<SOAR_FP32>(b, wg_absmax, wg, wg_search, params->method, lane_stream[lane]);
        i = j;
    }
    // always join, also after a failed launch, so that the caller's stream stays ordered
    if (lanes > 1 && !second->order(second->join, lane_stream[1], st)) result = SOAR_ERR_HIP;
    return result;
}

bool valid_mx_params(const soar_mx_params *p)
{
    if (!p || p->struct_size != sizeof(soar_mx_params)) return false;
    if (p->dss != 0 && p->dss != 1) return false;
    if (p->n_beta < 1 || p->n_beta > kMaxBeta) return false;
    if (!(p->beta_lo > 0.0f) || !(p->beta_hi >= p->beta_lo) || !(p->beta_hi < 1e30f)) return false;
    if (p->radius < 0 || p->radius > 127) return false;
    if (p->tiles_per_wg < 0 || p->tiles_per_wg > 65536 || (p->tiles_per_wg & (p->tiles_per_wg - 1))) return false;
    if (p->single_pass != 0 && p->single_pass != 1) return false;
    if (p->streams < 0 || p->streams > kLanes) return false;
    return true;
}

soar_status check_mx_shape(int64_t rows, int64_t cols, int64_t ld)
{
    if (rows <= 0 || cols <= 0 || cols % 32 != 0 || ld < cols) return SOAR_ERR_SHAPE;
    if (rows > (int64_t)1 << 31 || cols > (int64_t)1 << 31) return SOAR_ERR_SHAPE;
    if (rows * (cols / 32) > ((int64_t)1 << 31) - 16 * kWG) return SOAR_ERR_SHAPE;
    return SOAR_OK;
}

// ---- Eq. 3 / Eq. 4 on stored tensors: up to kGroupMax tensors of one element type and at most
// kStoredByteCap bytes of weights per launch
soar_status validate_stored(const soar_stored_desc &d, bool recon)
{
    if (!d.d_codes || !d.d_scales || !d.d_global_scale) return SOAR_ERR_NULL;
    if (recon ? (!d.d_w || !d.d_sse) : !d.d_out) return SOAR_ERR_NULL;
    if (d.dtype != SOAR_BF16 && d.dtype != SOAR_FP32) return SOAR_ERR_DTYPE;
    soar_status s = check_shape(d.rows, d.cols, d.ld_elems);
    if (s != SOAR_OK) return s;
    s = check_matrix_ptr(recon ? d.d_w : d.d_out, d.dtype, d.ld_elems);
    if (s != SOAR_OK) return s;
    if (reinterpret_cast<uintptr_t>(d.d_codes) % 8 != 0) return SOAR_ERR_ALIGN;
    return SOAR_OK;
}

// no pass follows that would find the group in the last-level cache: the cap only bounds the grid
constexpr int64_t kStoredByteCap = (int64_t)1 << 31;
int32_t stored_group_end(int32_t n, const soar_stored_desc *descs, int32_t i)
{
    int64_t bytes = 0;
    int32_t j = i;
    while (j < n && j - i < kGroupMax && descs[j].dtype == descs[i].dtype) {
        const int64_t b = descs[j].rows * descs[j].cols * (descs[j].dtype == SOAR_BF16 ? 2 : 4);
        if (j > i && bytes + b > kStoredByteCap) break;
        bytes += b;
        ++j;
    }
    return j;
}

soar_status run_stored_batch(int32_t n, const soar_stored_desc *descs, bool recon, hipStream_t st)
{
    if (n < 0) return SOAR_ERR_SHAPE;
    if (n > 0 && !descs) return SOAR_ERR_NULL;
    for (int32_t k = 0; k < n; ++k) {
        soar_status s = validate_stored(descs[k], recon);
        if (s != SOAR_OK) return s;
    }
    if (recon) {
        // all sums of the call first, kZeroMax per launch
        for (int32_t i = 0; i < n; i += kZeroMax) {
            ZeroBatch z;
            z.n = (uint32_t)(n - i < kZeroMax ? n - i : kZeroMax);
            for (uint32_t k = 0; k < z.n; ++k) z.sum[k] = descs[i + (int32_t)k].d_sse;
            hipLaunchKernelGGL(k_zero_sums, dim3(1), dim3(kZeroMax), 0, st, z);
            SOAR_LAUNCH_CHECK();
        }
    }
    for (int32_t i = 0; i < n;) {
        const int32_t j = stored_group_end(n, descs, i);
        StoredBatch b;
        std::memset(&b, 0, sizeof(b));
        b.n = (uint32_t)(j - i);
        uint32_t wg = 0;
        for (int32_t k = i; k < j; ++k) {
            const soar_stored_desc &d = descs[k];
            StoredTask &t = b.t[k - i];
            t.codes = d.d_codes; t.scales = d.d_scales; t.gscale = d.d_global_scale;
            t.w = d.d_w; t.out = d.d_out; t.sse = d.d_sse;
            t.ld = d.ld_elems;
            t.bpr = (uint32_t)(d.cols / 16);
            t.nblk = (uint32_t)(d.rows * (d.cols / 16));
            t.contiguous = d.ld_elems == d.cols ? 1u : 0u;
            const uint32_t per_wg = recon ? (uint32_t)kReconWG : (uint32_t)kWG;
            t.n_wg = (t.nblk + per_wg - 1) / per_wg;
            if (recon && t.n_wg > kReconGrid) t.n_wg = kReconGrid;
            t.wg_begin = wg;
            wg += t.n_wg;
        }
        const bool bf16 = descs[i].dtype == SOAR_BF16;
        ScopedTimer tm(recon ? SOAR_KERNEL_RECON : SOAR_KERNEL_DEQUANT, st);
        if (recon) {
            if (bf16) hipLaunchKernelGGL(k_recon<SOAR_BF16>, dim3(wg), dim3(kReconWG), 0, st, b);
            else hipLaunchKernelGGL(k_recon<SOAR_FP32>, dim3(wg), dim3(kReconWG), 0, st, b);
        } else {
            if (bf16) hipLaunchKernelGGL(k_dequant<SOAR_BF16>, dim3(wg), dim3(kWG), 0, st, b);
            else hipLaunchKernelGGL(k_dequant<SOAR_FP32>, dim3(wg), dim3(kWG), 0, st, b);
        }
        SOAR_LAUNCH_CHECK();
        i = j;
    }
    return SOAR_OK;
}

}  // namespace

// ------------------------------------------------------------------ C-ABI
extern "C" {

void soar_default_params(soar_params *p)
{
    if (!p) return;
    std::memset(p, 0, sizeof(*p));
    p->struct_size = sizeof(soar_params);
    p->method = SOAR_METHOD_SOAR;
    p->block = 16;
    p->iters = 1;
    p->dss_radius = 4;
    p->n_beta = 1;
    p->beta_lo = 1.0f;
    p->beta_hi = 1.0f;
    p->early_stop_rel = 1e-3f;
    p->search_mode = SOAR_SEARCH_AUTO;
    p->tiles_per_wg = 0;
    p->streams = 0;
    p->dd_mode = SOAR_DD_WINDOW;
    p->resident = SOAR_RESIDENT_AUTO;
    p->resident_wait_us = 0;
    p->tiles_per_wg_absmax = 0;
    p->tiles_per_wg_search = 0;
}

void soar_paper_params(soar_params *p)
{
    if (!p) return;
    soar_default_params(p);
    p->iters = 15;
    p->n_beta = 101;
    p->beta_lo = 0.5f;
    p->beta_hi = 1.5f;
    p->dd_mode = SOAR_DD_BRACKET;
    p->dss_radius = 1;
    p->early_stop_rel = 1e-3f;
}

size_t soar_workspace_bytes(int64_t rows, int64_t cols, const soar_params *params)
{
    if (!valid_params(params) || check_shape(rows, cols, cols) != SOAR_OK) return 0;
    return (size_t)kGroupMax * kSlotBytes + per_block_bytes(rows, cols);
}

size_t soar_batch_workspace_bytes(int32_t n, const soar_tensor_desc *descs, const soar_params *params)
{
    if (n <= 0 || !descs || !valid_params(params)) return 0;
    for (int32_t k = 0; k < n; ++k)
        if (check_shape(descs[k].rows, descs[k].cols, descs[k].ld_elems) != SOAR_OK) return 0;
    return batch_workspace_bytes(n, descs, params);
}

soar_status soar_quantize(const void *d_w, soar_dtype dtype, int64_t rows, int64_t cols, int64_t ld_elems,
                          const soar_params *params, uint8_t *d_codes, uint8_t *d_scales,
                          float *d_global_scale, double *d_sse, int32_t *d_status, void *d_workspace,
                          size_t workspace_bytes, void *hip_stream)
{
    soar_tensor_desc d;
    d.d_w = d_w;
    d.dtype = dtype;
    d.rows = rows;
    d.cols = cols;
    d.ld_elems = ld_elems;
    d.d_codes = d_codes;
    d.d_scales = d_scales;
    d.d_global_scale = d_global_scale;
    d.d_sse = d_sse;
    d.d_status = d_status;
    d.d_iters_run = nullptr;
    d.d_sse_trace = nullptr;
    d.d_amax_in = nullptr;
    return run_batch(1, &d, params, d_workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

soar_status soar_quantize_static(const void *d_w, soar_dtype dtype, int64_t rows, int64_t cols, int64_t ld_elems,
                                 const soar_params *params, uint8_t *d_codes, uint8_t *d_scales,
                                 float *d_global_scale, double *d_sse, int32_t *d_status, void *hip_stream)
{
    soar_tensor_desc d;
    d.d_w = d_w;
    d.dtype = dtype;
    d.rows = rows;
    d.cols = cols;
    d.ld_elems = ld_elems;
    d.d_codes = d_codes;
    d.d_scales = d_scales;
    d.d_global_scale = d_global_scale;
    d.d_sse = d_sse;
    d.d_status = d_status;
    d.d_iters_run = nullptr;
    d.d_sse_trace = nullptr;
    d.d_amax_in = nullptr;
    if (!params) return SOAR_ERR_NULL;
    soar_status s = validate_tensor(d, params);
    if (s != SOAR_OK) return s;
    if (rows * (cols / 16) > kStaticMaxBlocks) return SOAR_ERR_TOO_LARGE;
    void *ws = static_scratch_address();
    if (!ws) return SOAR_ERR_HIP;
    t_no_event_timing = true;
    s = run_batch(1, &d, params, ws, kStaticScratchBytes, static_cast<hipStream_t>(hip_stream));
    t_no_event_timing = false;
    return s;
}

soar_status soar_quantize_batch(int32_t n, const soar_tensor_desc *descs, const soar_params *params,
                                void *d_workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_batch(n, descs, params, d_workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

soar_status soar_dequantize_batch(int32_t n, const soar_stored_desc *descs, void *hip_stream)
{
    return run_stored_batch(n, descs, false, static_cast<hipStream_t>(hip_stream));
}

soar_status soar_recon_error_batch(int32_t n, const soar_stored_desc *descs, void *hip_stream)
{
    return run_stored_batch(n, descs, true, static_cast<hipStream_t>(hip_stream));
}

soar_status soar_dequantize(const uint8_t *d_codes, const uint8_t *d_scales, const float *d_global_scale,
                            int64_t rows, int64_t cols, soar_dtype out_dtype, void *d_out, int64_t ld_elems,
                            void *hip_stream)
{
    soar_stored_desc d;
    std::memset(&d, 0, sizeof(d));
    d.d_codes = d_codes; d.d_scales = d_scales; d.d_global_scale = d_global_scale;
    d.rows = rows; d.cols = cols; d.ld_elems = ld_elems;
    d.dtype = out_dtype;
    d.d_out = d_out;
    return run_stored_batch(1, &d, false, static_cast<hipStream_t>(hip_stream));
}

soar_status soar_recon_error(const void *d_w, soar_dtype dtype, int64_t rows, int64_t cols, int64_t ld_elems,
                             const uint8_t *d_codes, const uint8_t *d_scales, const float *d_global_scale,
                             double *d_sse, void *hip_stream)
{
    soar_stored_desc d;
    std::memset(&d, 0, sizeof(d));
    d.d_codes = d_codes; d.d_scales = d_scales; d.d_global_scale = d_global_scale;
    d.rows = rows; d.cols = cols; d.ld_elems = ld_elems;
    d.dtype = dtype;
    d.d_w = d_w;
    d.d_sse = d_sse;
    return run_stored_batch(1, &d, true, static_cast<hipStream_t>(hip_stream));
}

soar_status soar_e2m1_round_f32(const float *d_x, int64_t n, uint8_t *d_out, void *hip_stream)
{
    if (!d_x || !d_out) return SOAR_ERR_NULL;
    if (n < 0 || n > ((int64_t)1 << 38)) return SOAR_ERR_SHAPE;
    if (n == 0) return SOAR_OK;
    hipLaunchKernelGGL(k_e2m1_round, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), d_x, n, d_out);
    SOAR_LAUNCH_CHECK();
    return SOAR_OK;
}

soar_status soar_e4m3_project_f32(const float *d_x, int64_t n, uint8_t *d_out, void *hip_stream)
{
    if (!d_x || !d_out) return SOAR_ERR_NULL;
    if (n < 0 || n > ((int64_t)1 << 38)) return SOAR_ERR_SHAPE;
    if (n == 0) return SOAR_OK;
    hipLaunchKernelGGL(k_e4m3_project, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), d_x, n, d_out);
    SOAR_LAUNCH_CHECK();
    return SOAR_OK;
}

void soar_mx_default_params(soar_mx_params *p)
{
    if (!p) return;
    std::memset(p, 0, sizeof(*p));
    p->struct_size = sizeof(soar_mx_params);
    p->dss = 1;
    p->n_beta = 101;
    p->beta_lo = 0.5f;
    p->beta_hi = 1.5f;
    p->radius = 1;
    p->tiles_per_wg = 0;
    p->single_pass = 0;
    p->streams = 0;
}

size_t soar_mxfp4_workspace_bytes(int64_t rows, int64_t cols, const soar_mx_params *params)
{
    if (!valid_mx_params(params) || check_mx_shape(rows, cols, cols) != SOAR_OK) return 0;
    return kSlotBytes;
}

static int32_t mx_group_end(int32_t n, const soar_mx_tensor_desc *descs, int32_t i)
{
    auto bytes_of = [](const soar_mx_tensor_desc &d) { return d.rows * d.cols * (d.dtype == SOAR_BF16 ? 2 : 4); };
    int64_t bytes = bytes_of(descs[i]);
    int32_t j = i + 1;
    while (j < n && j - i < kGroupMax && descs[j].dtype == descs[i].dtype &&
           bytes + bytes_of(descs[j]) <= kOnePassByteCap) {
        bytes += bytes_of(descs[j]);
        ++j;
    }
    return j;
}

static int32_t mx_group_count(int32_t n, const soar_mx_tensor_desc *descs)
{
    int32_t groups = 0;
    for (int32_t i = 0; i < n; i = mx_group_end(n, descs, i)) ++groups;
    return groups;
}

soar_status soar_mxfp4_quantize_batch(int32_t n, const soar_mx_tensor_desc *descs, const soar_mx_params *params,
                                      void *d_workspace, size_t workspace_bytes, void *hip_stream)
{
    if (n < 0) return SOAR_ERR_SHAPE;
    if ((n > 0 && !descs) || !params) return SOAR_ERR_NULL;
    if (!valid_mx_params(params)) return SOAR_ERR_PARAM;
    for (int32_t k = 0; k < n; ++k) {
        const soar_mx_tensor_desc &d = descs[k];
        if (!d.d_w || !d.d_codes || !d.d_scales) return SOAR_ERR_NULL;
        if (d.dtype != SOAR_BF16 && d.dtype != SOAR_FP32) return SOAR_ERR_DTYPE;
        soar_status s = check_mx_shape(d.rows, d.cols, d.ld_elems);
        if (s != SOAR_OK) return s;
        s = check_matrix_ptr(d.d_w, d.dtype, d.ld_elems);
        if (s != SOAR_OK) return s;
        if (reinterpret_cast<uintptr_t>(d.d_codes) % 16 != 0) return SOAR_ERR_ALIGN;
    }
    if (n == 0) return SOAR_OK;
    if (!d_workspace || reinterpret_cast<uintptr_t>(d_workspace) % 256 != 0) return SOAR_ERR_WORKSPACE;
    const int32_t slots = n < kGroupMax ? n : kGroupMax;
    const int32_t groups = mx_group_count(n, descs);
    const int ws_lanes = groups > 1 ? kLanes : 1;
    if (workspace_bytes < (size_t)ws_lanes * slots * kSlotBytes) return SOAR_ERR_WORKSPACE;
    const int lanes = (groups > 1 && params->streams != 1) ? kLanes : 1;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *base = static_cast<char *>(d_workspace);
    // launch groups alternate between the caller's stream and one internal stream (forked and joined with
    // events), each with its own control slots, so that the ramp and the tail of one launch overlap another
    hipStream_t lane_stream[kLanes] = {st, st};
    SecondLane *second = nullptr;
    if (lanes > 1) {
        second = second_lane();
        if (!second) return SOAR_ERR_HIP;
        lane_stream[1] = second->stream;
    }
    soar_status result = SOAR_OK;
    {
        ScopedTimer tm(SOAR_KERNEL_INIT, st);
        hipLaunchKernelGGL(k_init, dim3(lanes * slots * kInitSplit), dim3(kWG), 0, st, base);
        if (hipGetLastError() != hipSuccess) result = SOAR_ERR_HIP;
    }
    if (lanes > 1 && result == SOAR_OK && !second->order(second->fork, st, lane_stream[1])) result = SOAR_ERR_HIP;
    const bool two_pass = params->dss && params->single_pass == 0 && params->n_beta >= 4 && params->n_beta <= kMaxListBeta;
    const size_t lds = ((size_t)params->n_beta * 4 + 255) / 256 * 256 + (two_pass ? (size_t)params->n_beta * kWG : 0);
    // consecutive tensors of one element type share a launch (up to kGroupMax); every kernel leaves the
    // control words of its slots as it found them, so the next group reuses them
    int32_t g = 0;
    for (int32_t i = 0; i < n && result == SOAR_OK; ++g) {
        const int32_t j = mx_group_end(n, descs, i);
        const int lane = g % lanes;
        char *lane_base = base + (size_t)lane * slots * kSlotBytes;
        hipStream_t lst = lane_stream[lane];
        MxBatch b;
        std::memset(&b, 0, sizeof(b));
        b.n = (uint32_t)(j - i);
        uint32_t wg = 0;
        int64_t group_tiles = 0;
        for (int32_t k = i; k < j; ++k) group_tiles += (descs[k].rows * (descs[k].cols / 32) + kWG - 1) / kWG;
        for (int32_t k = i; k < j; ++k) {
            const soar_mx_tensor_desc &d = descs[k];
            MxTask &t = b.t[k - i];
            t.w = d.d_w;
            t.codes = d.d_codes;
            t.scales = d.d_scales;
            t.sse = d.d_sse;
            t.status = d.d_status;
            t.ld = d.ld_elems;
            t.bpr = (uint32_t)(d.cols / 32);
            t.nblk = (uint32_t)(d.rows * (d.cols / 32));
            t.contiguous = d.ld_elems == d.cols ? 1u : 0u;
            const uint32_t tiles = (t.nblk + kWG - 1) / kWG;
            // the search is arithmetic-bound (see search_tiles_per_wg); the plain conversion streams
            uint32_t tpw = params->dss ? search_tiles_per_wg(group_tiles) : 2u;
            while (tpw > 1 && tpw > tiles) tpw >>= 1;
            if (params->tiles_per_wg) tpw = (uint32_t)params->tiles_per_wg;
            while ((tiles + tpw - 1) / tpw > (uint32_t)kMaxPartials) tpw <<= 1;
            t.tiles_per_wg = tpw;
            t.n_wg = (tiles + tpw - 1) / tpw;
            t.wg_begin = wg;
            wg += t.n_wg;
            char *slot = lane_base + (size_t)(k - i) * kSlotBytes;
            t.ctrl = reinterpret_cast<Ctrl *>(slot);
            t.counters = reinterpret_cast<uint32_t *>(slot + kCtrlBytes);
            t.part = reinterpret_cast<double *>(slot + kZeroedBytes);
            t.dss = params->dss;
            t.n_beta = params->n_beta;
            t.radius = params->radius;
            t.beta_lo = params->beta_lo;
            t.beta_hi = params->beta_hi;
            t.two_pass = two_pass ? 1 : 0;
        }
        ScopedTimer tm(SOAR_KERNEL_MX, lst);
        // the plain conversion is an instantiation of its own: it needs half the registers of the search
        const bool bf16 = descs[i].dtype == SOAR_BF16;
        if (params->dss) {
            if (bf16) hipLaunchKernelGGL((k_mx<SOAR_BF16, true>), dim3(wg), dim3(kWG), lds, lst, b);
            else hipLaunchKernelGGL((k_mx<SOAR_FP32, true>), dim3(wg), dim3(kWG), lds, lst, b);
        } else {
            if (bf16) hipLaunchKernelGGL((k_mx<SOAR_BF16, false>), dim3(wg), dim3(kWG), lds, lst, b);
            else hipLaunchKernelGGL((k_mx<SOAR_FP32, false>), dim3(wg), dim3(kWG), lds, lst, b);
        }
        if (hipGetLastError() != hipSuccess) result = SOAR_ERR_HIP;
        i = j;
    }
    // always join, also after a failed launch, so that the caller's stream stays ordered
    if (lanes > 1 && !second->order(second->join, lane_stream[1], st)) result = SOAR_ERR_HIP;
    return result;
}

size_t soar_mxfp4_batch_workspace_bytes(int32_t n, const soar_mx_tensor_desc *descs, const soar_mx_params *params)
{
    if (n <= 0 || !descs || !valid_mx_params(params)) return 0;
    for (int32_t k = 0; k < n; ++k)
        if (check_mx_shape(descs[k].rows, descs[k].cols, descs[k].ld_elems) != SOAR_OK) return 0;
    return (size_t)(mx_group_count(n, descs) > 1 ? kLanes : 1) * (size_t)(n < kGroupMax ? n : kGroupMax) * kSlotBytes;
}

soar_status soar_mxfp4_quantize(const void *d_w, soar_dtype dtype, int64_t rows, int64_t cols, int64_t ld_elems,
                                const soar_mx_params *params, uint8_t *d_codes, uint8_t *d_scales, double *d_sse,
                                int32_t *d_status, void *d_workspace, size_t workspace_bytes, void *hip_stream)
{
    soar_mx_tensor_desc d;
    d.d_w = d_w;
    d.dtype = dtype;
    d.rows = rows;
    d.cols = cols;
    d.ld_elems = ld_elems;
    d.d_codes = d_codes;
    d.d_scales = d_scales;
    d.d_sse = d_sse;
    d.d_status = d_status;
    return soar_mxfp4_quantize_batch(1, &d, params, d_workspace, workspace_bytes, hip_stream);
}

soar_status soar_mxfp4_dequantize_batch(int32_t n, const soar_stored_desc *descs, void *hip_stream)
{
    if (n < 0) return SOAR_ERR_SHAPE;
    if (n > 0 && !descs) return SOAR_ERR_NULL;
    for (int32_t k = 0; k < n; ++k) {
        const soar_stored_desc &d = descs[k];
        if (!d.d_codes || !d.d_scales || !d.d_out) return SOAR_ERR_NULL;
        if (d.dtype != SOAR_BF16 && d.dtype != SOAR_FP32) return SOAR_ERR_DTYPE;
        soar_status s = check_mx_shape(d.rows, d.cols, d.ld_elems);
        if (s != SOAR_OK) return s;
        s = check_matrix_ptr(d.d_out, d.dtype, d.ld_elems);
        if (s != SOAR_OK) return s;
        if (reinterpret_cast<uintptr_t>(d.d_codes) % 16 != 0) return SOAR_ERR_ALIGN;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    for (int32_t i = 0; i < n;) {
        const int32_t j = stored_group_end(n, descs, i);
        StoredBatch b;
        std::memset(&b, 0, sizeof(b));
        b.n = (uint32_t)(j - i);
        uint32_t wg = 0;
        for (int32_t k = i; k < j; ++k) {
            const soar_stored_desc &d = descs[k];
            StoredTask &t = b.t[k - i];
            t.codes = d.d_codes; t.scales = d.d_scales; t.out = d.d_out;
            t.ld = d.ld_elems;
            t.bpr = (uint32_t)(d.cols / 32);
            t.nblk = (uint32_t)(d.rows * (d.cols / 32));
            t.contiguous = d.ld_elems == d.cols ? 1u : 0u;
            t.n_wg = (t.nblk + kWG - 1) / kWG;
            t.wg_begin = wg;
            wg += t.n_wg;
        }
        ScopedTimer tm(SOAR_KERNEL_DEQUANT, st);
        if (descs[i].dtype == SOAR_BF16) hipLaunchKernelGGL(k_mx_dequant<SOAR_BF16>, dim3(wg), dim3(kWG), 0, st, b);
        else hipLaunchKernelGGL(k_mx_dequant<SOAR_FP32>, dim3(wg), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
        i = j;
    }
    return SOAR_OK;
}

soar_status soar_mxfp4_dequantize(const uint8_t *d_codes, const uint8_t *d_scales, int64_t rows, int64_t cols,
                                  soar_dtype out_dtype, void *d_out, int64_t ld_elems, void *hip_stream)
{
    soar_stored_desc d;
    std::memset(&d, 0, sizeof(d));
    d.d_codes = d_codes; d.d_scales = d_scales;
    d.rows = rows; d.cols = cols; d.ld_elems = ld_elems;
    d.dtype = out_dtype;
    d.d_out = d_out;
    return soar_mxfp4_dequantize_batch(1, &d, hip_stream);
}

soar_status soar_rcp_midrange_f32(const float *d_x, int64_t n, float *d_out, void *hip_stream)
{
    if (!d_x || !d_out) return SOAR_ERR_NULL;
    if (n < 0 || n > ((int64_t)1 << 38)) return SOAR_ERR_SHAPE;
    if (n == 0) return SOAR_OK;
    hipLaunchKernelGGL(k_rcp_midrange, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), d_x, n, d_out);
    SOAR_LAUNCH_CHECK();
    return SOAR_OK;
}

void soar_kernel_timing_enable(int enable)
{
    for (auto &v : g_timing.ev) {
        for (auto &p : v) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
        v.clear();
    }
    g_timing.enabled = enable != 0;
}

soar_status soar_kernel_timing_read(int kernel_id, double *total_ms, int64_t *launches)
{
    if (!total_ms || !launches) return SOAR_ERR_NULL;
    if (kernel_id < 0 || kernel_id >= SOAR_KERNEL_COUNT) return SOAR_ERR_PARAM;
    double sum = 0.0;
    for (auto &p : g_timing.ev[kernel_id]) {
        if (hipEventSynchronize(p.second) != hipSuccess) return SOAR_ERR_HIP;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, p.first, p.second) != hipSuccess) return SOAR_ERR_HIP;
        sum += ms;
    }
    *total_ms = sum;
    *launches = (int64_t)g_timing.ev[kernel_id].size();
    return SOAR_OK;
}

void soar_debug_arrival_plan(uint32_t n_workgroups, uint32_t workgroup, uint32_t out[3])
{
    if (!out || n_workgroups == 0 || workgroup >= n_workgroups) return;
    const ArrivalPlan p = arrival_plan(n_workgroups, workgroup);
    out[0] = p.ns;
    out[1] = p.slot;
    out[2] = p.expected;
}

soar_status soar_search_stats_enable(int enable)
{
    g_search_stats.store(false);
    if (enable) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(search_stats_words)) != hipSuccess) return SOAR_ERR_HIP;
        if (hipDeviceSynchronize() != hipSuccess || hipMemset(p, 0, sizeof(unsigned long long) * 4) != hipSuccess ||
            hipDeviceSynchronize() != hipSuccess)
            return SOAR_ERR_HIP;
        g_search_stats.store(true);
    }
    return SOAR_OK;
}

soar_status soar_search_stats_read(int64_t counts[4])
{
    if (!counts) return SOAR_ERR_NULL;
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(search_stats_words)) != hipSuccess) return SOAR_ERR_HIP;
    if (hipDeviceSynchronize() != hipSuccess) return SOAR_ERR_HIP;
    if (hipMemcpy(counts, p, sizeof(int64_t) * 4, hipMemcpyDeviceToHost) != hipSuccess) return SOAR_ERR_HIP;
    return SOAR_OK;
}

const char *soar_status_string(soar_status s)
{
    switch (s) {
    case SOAR_OK: return "ok";
    case SOAR_ERR_NULL: return "null pointer";
    case SOAR_ERR_SHAPE: return "bad shape";
    case SOAR_ERR_DTYPE: return "bad dtype";
    case SOAR_ERR_PARAM: return "bad parameter";
    case SOAR_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SOAR_ERR_HIP: return "HIP runtime error";
    case SOAR_ERR_ALIGN: return "misaligned pointer or leading dimension";
    case SOAR_ERR_TOO_LARGE: return "tensor larger than the built-in workspace of soar_quantize_static";
    }
    return "unknown status";
}

uint32_t soar_version(void) { return 0x00010000u; }

}  // extern "C"
