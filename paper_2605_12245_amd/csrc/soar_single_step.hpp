// The single-step path (Algorithm 1 with T = 1, beta = {1}): k_init, k_absmax (Eq. 1), k_stats
// (Eq. 1-2, 5) and k_search (Eq. 6, 8, packing); k_search also serves the plain conversion of Sec. 3.1.
#pragma once
#include "soar_device.hpp"

namespace {

// clears the control words, arrival counters and partial maxima of every slot
constexpr int kInitSplit = 8;             // workgroups per slot
static_assert(kZeroedBytes % 16 == 0, "control region is cleared with 16-byte stores");
__global__ __launch_bounds__(kWG) void k_init(char *slots_base)
{
    uint4 *p = reinterpret_cast<uint4 *>(slots_base + (size_t)(blockIdx.x / kInitSplit) * kSlotBytes);
    for (uint32_t k = (blockIdx.x % kInitSplit) * kWG + threadIdx.x; k < kZeroedBytes / 16; k += kInitSplit * kWG)
        p[k] = make_uint4(0u, 0u, 0u, 0u);
}

// max |w| over a tensor.  |bits| of finite floats order like the values; NaN
// and Inf patterns are larger than every finite one, so they surface in the max.
// For bf16 the running maximum stays packed (two 16-bit magnitudes per register,
// packed integer max) and is unpacked once per lane; for fp32 it is a plain max.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    u16x2 x, y;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    x = __builtin_elementwise_max(x, y);
    uint32_t r;
    __builtin_memcpy(&r, &x, 4);
    return r;
}

template <int DT>
__device__ __forceinline__ uint32_t absmax_accumulate(uint32_t m, uint4 v)
{
    if constexpr (DT == SOAR_BF16) {
        const uint32_t k = 0x7FFF7FFFu;
        return pk_max_u16(pk_max_u16(m, pk_max_u16(v.x & k, v.y & k)), pk_max_u16(v.z & k, v.w & k));
    } else {
        const uint32_t k = 0x7FFFFFFFu;
        return max(max(m, max(v.x & k, v.y & k)), max(v.z & k, v.w & k));
    }
}

template <int DT>
__global__ __launch_bounds__(kWG) void k_absmax(const Batch batch)
{
    __shared__ uint32_t s_wave[4];
    __shared__ uint32_t s_last;
    uint32_t lwg;
    const Task t = batch.t[find_task(batch, &Task::absmax, lwg)];
    const Shape sh = t.absmax;
    const uint32_t tid = threadIdx.x;
    constexpr int kChunks = DT == SOAR_BF16 ? 2 : 4;      // 16-byte pieces per block

    // tiles are dealt round-robin over the tensor's workgroups, so that at any moment
    // the workgroups in flight sweep one contiguous window of memory
    uint32_t m = 0;
    for (uint32_t k = 0; k < sh.tiles_per_wg; ++k) {
        const uint32_t i = (k * sh.n_wg + lwg) * kWG + tid;
        if (i >= t.nblk) break;
        const size_t off = block_offset(t, i) * (DT == SOAR_BF16 ? 2 : 4);
        const char *p = static_cast<const char *>(t.w) + off;
#pragma unroll
        for (int c = 0; c < kChunks; ++c) {
            const u32x4 v = load16<kStreamAbsmax>(p + 16 * c);
            m = absmax_accumulate<DT>(m, make_uint4(v.x, v.y, v.z, v.w));
        }
    }
    if constexpr (DT == SOAR_BF16) m = max(m & 0xFFFFu, m >> 16) << 16;
    m = wave_max_u32(m);
    if ((tid & 63) == 0) s_wave[tid >> 6] = m;
    __syncthreads();
    uint32_t *counters = t.counters;                       // kernel 0
    if (tid == 0) {
        m = max(max(s_wave[0], s_wave[1]), max(s_wave[2], s_wave[3]));
        const uint32_t ns = sh.n_wg < (uint32_t)kSlots ? sh.n_wg : (uint32_t)kSlots;
        // arrive_is_last waits for this read-modify-write to complete before it counts the workgroup in
        __hip_atomic_fetch_max(t.slot_max + (lwg % ns) * kSlotStride, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = arrive_is_last(counters, &t.ctrl->top[0], sh.n_wg, lwg) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    if (tid < 64) {
        uint32_t v = tid < kSlots ? __hip_atomic_load(t.slot_max + tid * kSlotStride, __ATOMIC_RELAXED,
                                                      __HIP_MEMORY_SCOPE_AGENT)
                                  : 0u;
        v = wave_max_u32(v);
        if (tid == 0) t.ctrl->amax_bits = v;
    }
    __syncthreads();
    if (tid < kSlots) t.slot_max[tid * kSlotStride] = 0u;
    reset_counters(counters, &t.ctrl->top[0]);
}

// Eq. 1-2 per block and the two tensor-wide sums of Eq. 5.  The per-block terms
// of kStage consecutive tiles are staged in LDS; lane t then folds the kStage
// adjacent terms t*kStage.. in registers and one wave tree finishes the group,
// which is the same adjacent-pair tree at a fraction of the cross-lane work.
// Each block's a/b -- or -Delta0 when its codes are all zero -- is kept for the
// search kernel.
template <int DT>
__global__ __launch_bounds__(kWG) void k_stats(const Batch batch)
{
    __shared__ double2 s_terms[kStage * kWG];
    __shared__ double s_wave[2][4];
    __shared__ double s_stack[2][32];
    __shared__ double s_tree[kWG];
    __shared__ uint32_t s_last;

    uint32_t lwg;
    const Task t = batch.t[find_task(batch, lwg)];
    const uint32_t tid = threadIdx.x;
    const uint32_t amax_bits = t.ctrl->amax_bits;
    const bool degenerate = amax_bits == 0u || amax_bits >= 0x7F800000u;
    const float alpha0 = f_of(amax_bits) / 2688.0f;
    const float alpha0_m = alpha0 * 6.0f;

    double wgN = 0.0, wgM = 0.0;
    const uint32_t tile0 = lwg * t.tiles_per_wg;
    const uint32_t T = t.tiles_per_wg < (uint32_t)kStage ? t.tiles_per_wg : (uint32_t)kStage;   // power of two
    for (uint32_t kg = 0; kg < t.tiles_per_wg; kg += T) {
        for (uint32_t kk = 0; kk < T; ++kk) {
            const uint32_t i = (tile0 + kg + kk) * kWG + tid;
            double tN = 0.0, tM = 0.0;
            if (i < t.nblk) {
                float rho = 0.0f;
                if (!degenerate) {
                    float w[16], q[16];
                    uint32_t nib[2], c0;
                    float delta0, a, b;
                    load_block<DT, kStreamStats>(t.w, block_offset(t, i), w);
                    block_init(w, alpha0, alpha0_m, c0, delta0, nib, q);
                    block_sums(w, q, a, b);
                    tN = (double)a * (double)delta0;
                    tM = ((double)b * (double)delta0) * (double)delta0;
                    rho = (b == 0.0f) ? -delta0 : a / b;      // first half of Eq. 6
                }
                __builtin_nontemporal_store(rho, t.rho + i);
            }
            s_terms[kk * kWG + tid] = make_double2(tN, tM);
        }
        __syncthreads();
        double vN, vM;
        {
            double2 t0 = s_terms[tid * T];
            vN = t0.x; vM = t0.y;
            if (T >= 2) {
                double2 t1 = s_terms[tid * T + 1];
                vN = vN + t1.x; vM = vM + t1.y;
            }
            if (T == 4) {
                double2 t2 = s_terms[tid * T + 2], t3 = s_terms[tid * T + 3];
                vN = vN + (t2.x + t3.x); vM = vM + (t2.y + t3.y);
            }
        }
        vN = wave_pair_tree(vN);
        vM = wave_pair_tree(vM);
        if ((tid & 63) == 0) { s_wave[0][tid >> 6] = vN; s_wave[1][tid >> 6] = vM; }
        __syncthreads();
        if (tid == 0) {
            // group sum, then binary-counter stack: group k closes every level whose bit of k is set
            vN = (s_wave[0][0] + s_wave[0][1]) + (s_wave[0][2] + s_wave[0][3]);
            vM = (s_wave[1][0] + s_wave[1][1]) + (s_wave[1][2] + s_wave[1][3]);
            const uint32_t k = kg / T;
            uint32_t lvl = 0;
            while ((k >> lvl) & 1u) {
                vN = s_stack[0][lvl] + vN;
                vM = s_stack[1][lvl] + vM;
                ++lvl;
            }
            s_stack[0][lvl] = vN;
            s_stack[1][lvl] = vM;
            wgN = vN; wgM = vM;          // after the last group: the sum of all tiles
        }
    }
    double *partN = t.part, *partM = t.part + kMaxPartials;
    uint32_t *counters = t.counters + 1 * kSlots * kSlotStride;
    if (tid == 0) {
        publish(partN + lwg, wgN);
        publish(partM + lwg, wgM);
        s_last = arrive_is_last(counters, &t.ctrl->top[1], t.n_wg, lwg) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    // last workgroup of the tensor: finish the trees and apply Eq. 5
    double NM[2];
    trees_of_partials<2>(t.part, t.n_wg, s_tree, &s_stack[0][0], NM);
    const double N = NM[0], M = NM[1];
    if (tid == 0) {
        float alpha1 = (M > 0.0) ? (float)(N / M) : alpha0;
        if (amax_bits == 0u) alpha1 = 1.0f;
        t.ctrl->alpha0 = alpha0;
        t.ctrl->alpha1 = alpha1;
        t.ctrl->N = N;
        t.ctrl->M = M;
        *t.gscale = alpha1;
    }
    reset_counters(counters, &t.ctrl->top[1]);
}

// Exhaustive form of the Eq. 8 search: candidates centre, -1, +1, -2, +2, ...;
// a later one wins only if strictly better.  A code outside [0x01, 0x7E] is
// clamped onto an already evaluated candidate and can then never win.
__device__ __forceinline__ void search_full(const float w[16], const float q[16], float alpha1, int centre,
                                            int radius, int &best, float &best_err)
{
    best = centre;
    best_err = block_error(w, q, alpha1 * e4m3_value((uint32_t)centre));
    for (int o = 1; o <= radius; ++o) {
        int cm = max(centre - o, (int)kE4M3Min);
        float em = block_error(w, q, alpha1 * e4m3_value((uint32_t)cm));
        if (em < best_err) { best_err = em; best = cm; }
        int cp = min(centre + o, (int)kE4M3Max);
        float ep = block_error(w, q, alpha1 * e4m3_value((uint32_t)cp));
        if (ep < best_err) { best_err = ep; best = cp; }
    }
}

// position of a candidate in the search order 0,-1,+1,-2,+2,...
__device__ __forceinline__ int search_rank(int code, int centre)
{
    const int o = code - centre;
    return o < 0 ? -2 * o - 1 : 2 * o;
}

// Certified short form of the same search.  For fixed codes the exact block
// error is a parabola in s = alpha*d, f(s) = A - 2Bs + Cs^2, with minimiser
// s* = B/C (B = sum w q, C = sum q^2).  The two window candidates that bracket
// s* are evaluated with the very same binary32 chain as the exhaustive search;
// their winner is the exhaustive winner provided that
//   (i)  the bracket really encloses s* (checked with a margin far above the
//        rounding error of the computed B/C), so that f rises monotonically
//        through every other candidate on either side, and
//   (ii) that rise, at least C*h^2 with h the E4M3 spacing (>= s/16), exceeds the
//        worst-case rounding error of the binary32 evaluation (18 ulp relative,
//        all terms being non-negative), so no unevaluated candidate can compute
//        to a value as small as the winner's.
// Where only one side of the bracket fails (i) -- s* within the margin of a candidate -- the next
// candidate on that side is evaluated as well and (i) is asked of the three.
// Returns false when a condition cannot be shown; the caller then runs the
// exhaustive search, so the result never depends on this shortcut.
__device__ __forceinline__ bool search_certified(const float w[16], const float q[16], float alpha1,
                                                 float inv_alpha1, int centre, int radius, int &best,
                                                 float &best_err)
{
    float B, C;
    block_sums(w, q, B, C);
    const int wmin = max(centre - radius, (int)kE4M3Min);
    const int wmax = min(centre + radius, (int)kE4M3Max);
    const float sstar = B * __builtin_amdgcn_rcpf(C);
    const float dstar = sstar * inv_alpha1;
    // largest E4M3 code whose value does not exceed dstar (approximately; (i) checks)
    const int lo_n = (int)(__float_as_uint(dstar) >> 20) - (120 << 3);
    const int lo_s = (int)(dstar * 512.0f);
    const int lo = dstar >= 0x1p-6f ? lo_n : lo_s;
    const int ka = min(max(lo, wmin), wmax);
    const int kb = min(max(lo + 1, wmin), wmax);
    const float sa = alpha1 * e4m3_value((uint32_t)ka);
    const float sb = alpha1 * e4m3_value((uint32_t)kb);
    const float fa = block_error(w, q, sa);
    const float fb = block_error(w, q, sb);
    // ka <= kb <= ka + 1.  In the order 0,-1,+1,-2,+2,... the upper of two adjacent codes comes
    // first exactly when the lower one lies below the centre.
    const bool b_wins = (fb < fa) || (fb == fa && ka < centre);
    best = b_wins ? kb : ka;
    best_err = b_wins ? fb : fa;
    const bool left_ok = (ka == wmin) || (sa * (1.0f + 0x1p-17f) <= sstar);
    const bool right_ok = (kb == wmax) || (sb * (1.0f - 0x1p-17f) >= sstar);
    bool enclosed = left_ok && right_ok;
    if (left_ok != right_ok) {
        // s* sits within the margin of one of the two candidates (about two blocks in ten thousand), so that
        // side of the bracket is in doubt: the next candidate on that side, a whole E4M3 step further out,
        // settles it -- the three enclose s* if it lies clear of s* in its turn.  Its rank in the search
        // order decides ties as in the exhaustive loop.
        const int ke = left_ok ? kb + 1 : ka - 1;            // inside the window: the side in doubt is not at its edge
        const float se = alpha1 * e4m3_value((uint32_t)ke);
        const float fe = block_error(w, q, se);
        enclosed = left_ok ? (ke == wmax) || (se * (1.0f - 0x1p-17f) >= sstar)
                           : (ke == wmin) || (se * (1.0f + 0x1p-17f) <= sstar);
        if (fe < best_err || (fe == best_err && search_rank(ke, centre) < search_rank(best, centre))) {
            best = ke;
            best_err = fe;
        }
    }
    const bool margin_ok = best_err < 512.0f * (C * (sa * sa));
    const bool range_ok = (B > 0x1p-100f) && (best_err > 0x1p-100f) && (C > 0.0f);
    return enclosed && margin_ok && range_ok;
}

// Diagnostics (off unless the host asks): how often the certified search had to hand over to the
// exhaustive one.  stats[0] blocks searched, [1] blocks that fell back, [2] wave steps (one block per lane),
// [3] wave steps in which at least one lane fell back (the whole wave then waits for the exhaustive loop).
__device__ __forceinline__ void count_search(unsigned long long *stats, bool certified)
{
    const unsigned long long active = __builtin_amdgcn_ballot_w64(true);
    const unsigned long long fell = __builtin_amdgcn_ballot_w64(!certified);
    if ((threadIdx.x & 63u) == (uint32_t)__builtin_ctzll(active)) {
        atomicAdd(stats + 0, (unsigned long long)__builtin_popcountll(active));
        atomicAdd(stats + 1, (unsigned long long)__builtin_popcountll(fell));
        atomicAdd(stats + 2, 1ull);
        atomicAdd(stats + 3, fell != 0ull ? 1ull : 0ull);
    }
}

// Eq. 6, projection, new assignment, Eq. 8 search, packing, error sum.
// METHOD RTN emits the Eq. 1-2 state instead.
// (bf16: held to 64 registers, eight waves per SIMD; left to itself the compiler takes 83 for a shorter schedule and loses more in
// occupancy than it gains)
template <int DT, int METHOD>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(DT == SOAR_BF16 ? 8 : 4))) void k_search(const Batch batch)
{
    __shared__ double s_wave[4];
    __shared__ double s_tree[kWG];
    __shared__ double s_stack[16];
    __shared__ uint32_t s_last;
    // The coalescing exchange pays where the reads bound the kernel: binary32 input (64 bytes per lane)
    // and the plain conversion.  The bf16 search is as much bound by its arithmetic and gains nothing.
    constexpr bool kExchange = DT == SOAR_FP32 || METHOD == SOAR_METHOD_RTN;
    constexpr int kP = pieces_per_block<DT, 16>();
    __shared__ u32x4 s_x[kExchange ? kWG * kP : 1];    // load_wave_blocks: one region per wave

    uint32_t lwg;
    const Task t = batch.t[find_task(batch, &Task::search, lwg)];
    const Shape sh = t.search;
    const uint32_t tid = threadIdx.x;
    const int radius = batch.radius;
    const bool full_search = batch.full_search != 0;
    // a supplied maximum that is unusable is read as NaN: the arithmetic below stays defined,
    // the outputs are unspecified and the status says why
    bool bad_amax = false;
    uint32_t amax_bits = t.ctrl->amax_bits;
    if (METHOD == SOAR_METHOD_RTN && t.amax_in) {
        const float given = *t.amax_in;
        bad_amax = !(given > 0.0f) || __float_as_uint(given) >= 0x7F800000u;
        amax_bits = bad_amax ? 0x7FC00000u : __float_as_uint(given);
    }
    const bool allzero = amax_bits == 0u;
    const float alpha0 = f_of(amax_bits) / 2688.0f;
    const float alpha0_m = alpha0 * 6.0f;
    const float alpha1 = (METHOD == SOAR_METHOD_SOAR) ? t.ctrl->alpha1 : alpha0;
    const float inv_alpha1 = __builtin_amdgcn_rcpf(alpha1);

    // tiles dealt round-robin over the tensor's workgroups (see k_absmax)
    double sse = 0.0;
    for (uint32_t k = 0; k < sh.tiles_per_wg; ++k) {
        const uint32_t i = (k * sh.n_wg + lwg) * kWG + tid;
        float w[16], q[16];
        uint32_t nib[2];
        if (kExchange && t.contiguous) {
            // packed rows: the wave reads its 64 blocks coalesced (all of its lanes take part)
            const uint32_t wave_first = i - (tid & 63u);
            if (wave_first >= t.nblk) break;
            load_wave_blocks<DT, 16, kStreamSearch>(t.w, wave_first, t.nblk, s_x + (tid >> 6) * (64 * kP), w);
            if (i >= t.nblk) break;
        } else {
            if (i >= t.nblk) break;
            load_block<DT, kStreamSearch>(t.w, block_offset(t, i), w);
        }
        uint32_t out_code;
        float out_err;
        if (allzero) {
            // every weight is +-0: smallest scale, zero codes carrying the sign
            float x[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) x[j] = w[j];
            nib[0] = fp4x8(x);
            nib[1] = fp4x8(x + 8);
            out_code = kE4M3Min;
            out_err = 0.0f;
        } else if constexpr (METHOD == SOAR_METHOD_RTN) {
            uint32_t c0;
            float delta0;
            block_init(w, alpha0, alpha0_m, c0, delta0, nib, q);
            out_code = c0;
            out_err = block_error(w, q, alpha0 * delta0);
        } else {
            const float rho = __builtin_nontemporal_load(t.rho + i);                // a / b >= 0, or -Delta0 where b == 0
            const float delta_star = (rho < 0.0f) ? -rho : rho / alpha1;
            const int centre = (int)e4m3_project(delta_star);
            assign_codes(w, alpha1 * delta_star, nib, q);
            int best;
            float best_err;
            bool done = false;
            if (!full_search) {
                done = search_certified(w, q, alpha1, inv_alpha1, centre, radius, best, best_err);
                if (batch.search_stats) count_search(batch.search_stats, done);
            }
            if (!done) search_full(w, q, alpha1, centre, radius, best, best_err);
            out_code = (uint32_t)best;
            out_err = best_err;
        }
        {
            // streaming stores: the outputs are not read again by this path
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            u32x2 packed = {nib[0], nib[1]};
            __builtin_nontemporal_store(packed, reinterpret_cast<u32x2 *>(t.codes) + i);
            __builtin_nontemporal_store((uint8_t)out_code, t.scales + i);
        }
        sse += (double)out_err;
    }
    // error sum: fixed order for a given launch shape
    sse = wave_pair_tree(sse);
    if ((tid & 63) == 0) s_wave[tid >> 6] = sse;
    __syncthreads();
    double *partS = t.part + 2 * kMaxPartials;
    uint32_t *counters = t.counters + 2 * kSlots * kSlotStride;
    if (tid == 0) {
        publish(partS + lwg, (s_wave[0] + s_wave[1]) + (s_wave[2] + s_wave[3]));
        s_last = arrive_is_last(counters, &t.ctrl->top[2], sh.n_wg, lwg) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    double total;
    trees_of_partials<1>(partS, sh.n_wg, s_tree, s_stack, &total);
    if (tid == 0) {
        if (t.sse) *t.sse = total;
        if (t.status)
            *t.status = bad_amax ? SOAR_STATUS_BAD_AMAX
                                 : (amax_bits >= 0x7F800000u ? SOAR_STATUS_NONFINITE : 0) | (allzero ? SOAR_STATUS_ALLZERO : 0);
        if (METHOD == SOAR_METHOD_RTN) *t.gscale = allzero ? 1.0f : alpha0;
    }
    reset_counters(counters, &t.ctrl->top[2]);
}

// ------------------------------------------------------------------ one launch, the tensor resident on chip
// A tensor handed over alone pays, on the three-pass path, four dependent launches whose ramp and tail
// dominate below a few hundred MiB, and reads its weights three times.  k_resident does the whole
// single-step path in ONE launch of at most one workgroup per compute unit: every lane loads its (up to
// kResMaxPer) blocks once and keeps them in registers as loaded; the two tensor-wide results (the Eq. 1
// maximum, the Eq. 5 sums) cross the grid through words in the workspace; the search then runs from the
// registers.  The weights are read once (2 + 9/16 bytes per bf16 weight instead of 6 + 9/16).
//
// Workgroup g owns the L * R consecutive blocks from g * L * R on (an aligned power of two, so its partial
// sums are nodes of the adjacent-pair tree) and a wave 64 R consecutive ones, in "packets" of up to 128
// bytes of weights per lane: a lane owns ADJACENT blocks (4 bf16 or 2 fp32 blocks per packet; with four
// fp32 blocks per lane a wave's range is two packets).  So the first levels of the tree are additions in
// registers, one DPP wave tree covers a packet of the whole wave, the L/64 wave sums, in block order, go
// through the wave tree once more, and a lane's scale bytes and code bytes leave in one or two stores.
// Packed rows are read through the coalescing wave exchange (load_wave_pieces).  Across workgroups the tree continues over groups of 64 consecutive workgroups (one wave
// tree, a workgroup per lane) and then over the at most 4 groups.  Same arithmetic, same trees as the
// three-pass path: identical bytes.
//
// Crossing the grid.  All workgroups of the launch must be on the machine at the same time (the host
// launches at most one per compute unit and takes the three-pass path otherwise).  A trip through memory
// from one workgroup to another takes about 1.4 us on this part, and 256 workgroups that each read all
// 256 results queue for several microseconds more, so:
//  - there is no counter and no separate "ready" flag, hence no word that has to be cleared beforehand and
//    no second trip for the value: every word a workgroup publishes (an agent-scope atomic store) carries
//    the launch's TOKEN beside its payload, and a reader accepts a word only with that token.  A binary64
//    sum travels as three words of 22 payload bits and 42 token bits; the first crossing's word holds the
//    bf16 / fp32 maximum in 15 / 31 bits beside 49 / 33 token bits.  The token is `nonce ^ epoch * odd`:
//    the nonce comes from the host (new for every call), the epoch from the workspace, advanced by the
//    launch itself once every workgroup has read it (workgroup 0, after the first crossing), so that a
//    replayed HIP graph -- same kernel arguments -- still sees a new token every time.  Memory the library
//    never wrote matches a token field with probability 2^-42 (2^-33) per word;
//  - up to 64 workgroups read each other's words directly (one trip); above that the first workgroup of
//    every group of 64 gathers its group and publishes the group's result, and everybody gathers the at
//    most 4 group results (two trips, little traffic); the error sum, which only workgroup 0 needs, is
//    gathered by workgroup 0 alone in one trip.
// Every wait is BOUNDED: a workgroup whose time is up publishes the complemented token in its words (so
// that the others leave at once instead of waiting out the limit), sets SOAR_STATUS_GAVE_UP and returns;
// every wave of the grid then reaches its end.
constexpr int kResMaxWG = 256;            // workgroups of one launch, at most
constexpr int kResMaxPer = 4;             // blocks per lane, at most
constexpr int kResGroup = 64;             // workgroups per group: a wave gathers one with a workgroup per lane
constexpr int kResGroups = kResMaxWG / kResGroup;
constexpr uint64_t kResOdd = 0x9E3779B97F4A7C15ull;
constexpr int kResSumBits = 22;           // payload bits of a word that carries a third of a binary64 value
// Places inside Task::part, in 8-byte words.  First level: per kind of word kResMaxWG entries (one per
// workgroup).  Second level: kResGroups entries (one per group) per kind, in kResCopies copies
// kResCopyStride words apart: every workgroup polls the second level, and a few lines polled by 250
// workgroups at once queue at their memory channel (the publisher's stores behind them); a reader polls
// the copy of its own number modulo kResCopies.
constexpr int kResCopies = 8;
constexpr uint32_t kResCopyStride = 544;                                          // 17 * 256 bytes
constexpr uint32_t kResMax1 = 0;                                                  // 1 kind: token | maximum
constexpr uint32_t kResNM1 = 512;                                                 // 6 kinds: N and M in thirds
constexpr uint32_t kResErr1 = 2304;                                               // 3 kinds: the error sum in thirds
constexpr uint32_t kResMax2 = 3072, kResNM2 = kResMax2 + kResCopies * kResCopyStride;
static_assert(kResMax1 + kResMaxWG <= kResNM1 && kResNM1 + 6 * kResMaxWG <= kResErr1 && kResErr1 + 3 * kResMaxWG <= kResMax2 &&
              6 * kResGroups <= kResCopyStride && kResNM2 + kResCopies * kResCopyStride <= 3 * kMaxPartials,
              "layout of the crossing words");
constexpr uint32_t kResDirect = 16;       // up to this many workgroups read each other's words directly

struct ResidentArgs {
    int32_t  radius, full_search;
    uint64_t nonce;                       // new for every call
    uint64_t wait_ticks;                  // bound of the waits of a workgroup together, in ticks of the wall clock
    unsigned long long *search_stats;     // null, or the diagnostic counters of count_search
};

// what wave 0 of a workgroup needs for its crossings
struct ResidentGrid {
    uint32_t g, G;
    uint64_t tok, t0, ticks;
    uint64_t *words;                      // Task::part
};

// The bound of a wait: the wall clock (100 MHz on this part), and -- should that clock ever stand still -- a
// number of polling rounds that takes several times as long (a round is at least one trip to memory).
__device__ __forceinline__ bool resident_time_is_up(const ResidentGrid &r, uint64_t round)
{
    return (uint64_t)wall_clock64() - r.t0 > r.ticks || round > 1024ull + r.ticks / 8ull;
}

// one lane: NW kinds of words for entry e; kind w of entry e sits at dst[w * stride + e]
template <int NW, int PBITS>
__device__ __forceinline__ void resident_publish(uint64_t *dst, uint32_t stride, uint32_t e, uint64_t tok, const uint64_t pay[NW])
{
#pragma unroll
    for (int w = 0; w < NW; ++w)
        __hip_atomic_store(dst + w * stride + e, (tok << PBITS) | pay[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// wave 0, all lanes: a group's result into every copy of the second level (lane c writes copy c)
template <int NW, int PBITS>
__device__ __forceinline__ void resident_publish_copies(uint64_t *dst, uint32_t grp, uint64_t tok, const uint64_t pay[NW])
{
    const uint32_t lane = threadIdx.x & 63u;
    if (lane < (uint32_t)kResCopies) resident_publish<NW, PBITS>(dst + lane * kResCopyStride, kResGroups, grp, tok, pay);
}

// Wave 0, all lanes: wait until entries first .. first + count - 1 (count <= 64 * K) of all NW kinds carry the
// token; lane l then holds the payloads of entries first + l + 64 k in pay[k][.] (zeros from `count` on).
// False when somebody has given up (a word with the complemented token) or the time is up.
template <int NW, int PBITS, int K>
__device__ __forceinline__ bool resident_gather(const ResidentGrid &r, const uint64_t *src, uint32_t stride, uint32_t first,
                                                uint32_t count, uint64_t pay[K][NW])
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t want = (r.tok << PBITS) >> PBITS, gone_field = (~r.tok << PBITS) >> PBITS;
    for (uint64_t round = 0;; ++round) {
        bool pending = false, gone = false;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const uint32_t e = lane + 64u * (uint32_t)k;
#pragma unroll
            for (int w = 0; w < NW; ++w) pay[k][w] = 0ull;
            if (e < count) {
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const uint64_t v = __hip_atomic_load(src + w * stride + first + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const uint64_t field = v >> PBITS;
                    gone = gone || field == gone_field;
                    pending = pending || field != want;
                    pay[k][w] = v & ((1ull << PBITS) - 1ull);
                }
            }
        }
        if (__builtin_amdgcn_ballot_w64(gone) != 0ull) return false;
        if (__builtin_amdgcn_ballot_w64(pending) == 0ull) return true;
        if (resident_time_is_up(r, round)) return false;
    }
}

// Wave 0, all lanes: the maximum of `value` over the grid (uniform on return).
template <int PBITS>
__device__ __forceinline__ bool resident_cross_max(const ResidentGrid &r, uint32_t &value)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t grp = r.g / kResGroup, groups = (r.G + kResGroup - 1) / kResGroup;
    uint64_t pay[1][1] = {{value}};
    if (lane == 0) resident_publish<1, PBITS>(r.words + kResMax1, kResMaxWG, r.g, r.tok, pay[0]);
    if (r.G > kResDirect) {
        if (r.g % kResGroup == 0u) {
            if (!resident_gather<1, PBITS, 1>(r, r.words + kResMax1, kResMaxWG, grp * kResGroup,
                                              min((uint32_t)kResGroup, r.G - grp * kResGroup), pay)) return false;
            pay[0][0] = wave_max_u32((uint32_t)pay[0][0]);
            resident_publish_copies<1, PBITS>(r.words + kResMax2, grp, r.tok, pay[0]);
        }
        if (!resident_gather<1, PBITS, 1>(r, r.words + kResMax2 + (r.g % kResCopies) * kResCopyStride, kResGroups, 0u, groups, pay))
            return false;
    } else if (!resident_gather<1, PBITS, 1>(r, r.words + kResMax1, kResMaxWG, 0u, r.G, pay)) {
        return false;
    }
    value = wave_max_u32((uint32_t)pay[0][0]);
    return true;
}

__device__ __forceinline__ void resident_split(double v, uint64_t pay[3])
{
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    pay[0] = b & ((1ull << kResSumBits) - 1ull);
    pay[1] = (b >> kResSumBits) & ((1ull << kResSumBits) - 1ull);
    pay[2] = b >> (2 * kResSumBits);
}

__device__ __forceinline__ double resident_join(const uint64_t pay[3])
{
    return __longlong_as_double((long long)(pay[0] | pay[1] << kResSumBits | pay[2] << (2 * kResSumBits)));
}

// Wave 0, all lanes, every workgroup: the adjacent-pair tree sums of NV binary64 values (one set per
// workgroup, in workgroup order, zero-padded) over the grid; uniform on return.
template <int NV>
__device__ __forceinline__ bool resident_cross_sums(const ResidentGrid &r, uint32_t at1, uint32_t at2, double v[NV])
{
    constexpr int NW = 3 * NV, P = kResSumBits;
    static_assert(NW * kResGroups <= (int)kResCopyStride, "a copy holds every kind");
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t grp = r.g / kResGroup, groups = (r.G + kResGroup - 1) / kResGroup;
    uint64_t pay[1][NW];
    auto split = [&]() {
#pragma unroll
        for (int n = 0; n < NV; ++n) resident_split(v[n], &pay[0][3 * n]);
    };
    auto tree = [&]() {                   // lane e holds entry e
#pragma unroll
        for (int n = 0; n < NV; ++n) v[n] = wave_pair_tree(resident_join(&pay[0][3 * n]));
    };
    split();
    if (lane == 0) resident_publish<NW, P>(r.words + at1, kResMaxWG, r.g, r.tok, pay[0]);
    if (r.G > kResDirect) {
        if (r.g % kResGroup == 0u) {
            if (!resident_gather<NW, P, 1>(r, r.words + at1, kResMaxWG, grp * kResGroup,
                                           min((uint32_t)kResGroup, r.G - grp * kResGroup), pay)) return false;
            tree();
            split();
            resident_publish_copies<NW, P>(r.words + at2, grp, r.tok, pay[0]);
        }
        if (!resident_gather<NW, P, 1>(r, r.words + at2 + (r.g % kResCopies) * kResCopyStride, kResGroups, 0u, groups, pay))
            return false;
    } else if (!resident_gather<NW, P, 1>(r, r.words + at1, kResMaxWG, 0u, r.G, pay)) {
        return false;
    }
    tree();
    return true;
}

// Wave 0, all lanes: the same sum of ONE value, wanted by workgroup 0 only, which gathers all workgroups in
// one trip (lane l holds workgroups l, l + 64, ...: the tree of a group is a wave tree, the groups follow);
// the other workgroups return as soon as they have published.
__device__ __forceinline__ bool resident_collect_sum(const ResidentGrid &r, uint32_t at1, double &v)
{
    const uint32_t lane = threadIdx.x & 63u;
    uint64_t pay[kResGroups][3];
    resident_split(v, pay[0]);
    if (lane == 0) resident_publish<3, kResSumBits>(r.words + at1, kResMaxWG, r.g, r.tok, pay[0]);
    if (r.g != 0u) return true;
    if (!resident_gather<3, kResSumBits, kResGroups>(r, r.words + at1, kResMaxWG, 0u, r.G, pay)) return false;
    double s[kResGroups];
#pragma unroll
    for (int k = 0; k < kResGroups; ++k) s[k] = wave_pair_tree(resident_join(pay[k]));
    static_assert(kResGroups == 4, "the tree over the groups is written out");
    v = (s[0] + s[1]) + (s[2] + s[3]);
    return true;
}

template <int DT, int METHOD, int L, int R>
__global__ __launch_bounds__(L) void k_resident(const Task t, const ResidentArgs args)
{
    static_assert(L == 256 || L == 1024, "workgroup of 4 or 16 waves");
    static_assert(R == 1 || R == 2 || R == 4, "blocks per lane");
    constexpr int kWaves = L / 64;
    constexpr int kParts = kWaves;                           // wave sums of a workgroup, in block order
    constexpr int kP = pieces_per_block<DT, 16>();
    constexpr int kX = R * kP <= 8 ? R : 8 / kP;             // adjacent blocks of a lane in one packet (<= 128 bytes)
    constexpr int kPackets = R / kX;                         // 1 or 2
    constexpr int kXP = kX * kP;                             // 16-byte pieces of a lane per packet: 2, 4 or 8
    static_assert(kPackets == 1 || kPackets == 2, "packets of a wave");
    __shared__ u32x4 s_x[kWaves * 64 * kXP];                 // load_wave_pieces: one region per wave
    // first crossing: bf16 maxima have 15 significant bits (sign cleared, low half zero), fp32 ones 31
    constexpr int kMaxBits = DT == SOAR_BF16 ? 15 : 31;
    __shared__ uint32_t s_max[kWaves];
    __shared__ double s_part[3][kParts];
    __shared__ float s_alpha1;
    __shared__ uint32_t s_amax, s_gone;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t wave_first = (blockIdx.x * (uint32_t)L + wave * 64u) * (uint32_t)R;   // first block of this wave
    // block k (0 .. R-1) of this lane: packet k / kX of the wave, there the lane's kX adjacent blocks
    auto blk = [&](int k) -> uint32_t {
        return wave_first + (uint32_t)(k / kX) * (64u * kX) + lane * (uint32_t)kX + (uint32_t)(k % kX);
    };
    uint64_t *epoch_p = &t.ctrl->epoch;

    ResidentGrid grid;
    grid.g = blockIdx.x;
    grid.G = gridDim.x;
    grid.tok = 0;
    grid.t0 = 0;
    grid.ticks = args.wait_ticks;
    grid.words = reinterpret_cast<uint64_t *>(t.part);
    uint64_t epoch = 0;
    if (grid.G > 1u) {
        epoch = __hip_atomic_load(epoch_p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        grid.tok = args.nonce ^ (epoch * kResOdd);
        grid.t0 = (uint64_t)wall_clock64();
    }
    // one lane: leave the launch and tell the others -- whoever gathers this workgroup's words, now or at a
    // later crossing, finds the complemented token in the first of them
    auto give_up = [&]() {
        const uint64_t gone = ~grid.tok << kResSumBits, gone_max = ~grid.tok << kMaxBits;
        __hip_atomic_store(grid.words + kResMax1 + grid.g, gone_max, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(grid.words + kResNM1 + grid.g, gone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(grid.words + kResErr1 + grid.g, gone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (grid.g % kResGroup == 0u) {
            for (int c = 0; c < kResCopies; ++c) {
                __hip_atomic_store(grid.words + kResMax2 + c * kResCopyStride + grid.g / kResGroup, gone_max, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(grid.words + kResNM2 + c * kResCopyStride + grid.g / kResGroup, gone, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // any change of the epoch will do for the next launch
        __hip_atomic_fetch_add(epoch_p, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (t.status) *t.status = SOAR_STATUS_GAVE_UP;
    };

    // ---- the blocks of this lane, as loaded; Eq. 1 maximum
    u32x4 raw[R][kP];
    uint32_t m = 0;
    if (t.contiguous) {
        // packed rows: the wave reads each packet's range in coalesced 16-byte pieces (all of its lanes take part)
#pragma unroll
        for (int pk = 0; pk < kPackets; ++pk) {
            const uint32_t first = wave_first + (uint32_t)pk * (64u * kX);
            const uint32_t have = first < t.nblk ? min(64u * kX, t.nblk - first) * (uint32_t)kP : 0u;
            u32x4 v[kXP];
            load_wave_pieces<kXP, true>(static_cast<const u32x4 *>(t.w) + (size_t)first * kP, have, s_x + wave * (64 * kXP), v);
#pragma unroll
            for (int q = 0; q < kXP; ++q) raw[pk * kX + q / kP][q % kP] = v[q];
        }
    } else {
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const uint32_t i = blk(k);
#pragma unroll
            for (int p = 0; p < kP; ++p) raw[k][p] = u32x4{0u, 0u, 0u, 0u};
            if (i < t.nblk) {
                const char *src = static_cast<const char *>(t.w) + block_offset(t, i) * (DT == SOAR_BF16 ? 2 : 4);
#pragma unroll
                for (int p = 0; p < kP; ++p) raw[k][p] = load16<false>(src + 16 * p);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < R; ++k)
#pragma unroll
        for (int p = 0; p < kP; ++p)
            m = absmax_accumulate<DT>(m, make_uint4(raw[k][p].x, raw[k][p].y, raw[k][p].z, raw[k][p].w));
    if constexpr (DT == SOAR_BF16) m = max(m & 0xFFFFu, m >> 16) << 16;
    m = wave_max_u32(m);
    if (lane == 0) s_max[wave] = m;
    __syncthreads();
    if (wave == 0) {
        uint32_t amax = wave_max_u32(lane < (uint32_t)kWaves ? s_max[lane] : 0u);
        bool ok = true;
        if (grid.G > 1u) {
            uint32_t value = DT == SOAR_BF16 ? amax >> 16 : amax;
            ok = resident_cross_max<kMaxBits>(grid, value);
            amax = DT == SOAR_BF16 ? value << 16 : value;
            if (lane == 0) {
                if (!ok) give_up();
                else if (grid.g == 0u)     // every workgroup has read the epoch by now: the next launch gets a new token
                    __hip_atomic_store(epoch_p, epoch + 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (lane == 0) { s_amax = amax; s_gone = ok ? 0u : 1u; }
    }
    __syncthreads();
    if (s_gone) return;
    const uint32_t amax_bits = s_amax;
    const bool allzero = amax_bits == 0u;
    const bool degenerate = allzero || amax_bits >= 0x7F800000u;
    const float alpha0 = f_of(amax_bits) / 2688.0f;
    const float alpha0_m = alpha0 * 6.0f;

    auto widen = [&](int k, float w[16]) {
        if constexpr (DT == SOAR_BF16) {
#pragma unroll
            for (int p = 0; p < kP; ++p) {
                const uint32_t u[4] = {raw[k][p].x, raw[k][p].y, raw[k][p].z, raw[k][p].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    w[8 * p + 2 * e] = f_of(u[e] << 16);
                    w[8 * p + 2 * e + 1] = f_of(u[e] & 0xFFFF0000u);
                }
            }
        } else {
#pragma unroll
            for (int p = 0; p < kP; ++p) {
                w[4 * p] = f_of(raw[k][p].x); w[4 * p + 1] = f_of(raw[k][p].y);
                w[4 * p + 2] = f_of(raw[k][p].z); w[4 * p + 3] = f_of(raw[k][p].w);
            }
        }
    };
    // one binary64 term per block of the lane: the adjacent-pair tree over the lane's blocks of a packet in
    // registers, over the packet with the wave tree, over the packets; the wave sum goes to its place in block order
    auto wave_sum_to_lds = [&](int which, const double term[R]) {
        double v[kPackets];
#pragma unroll
        for (int pk = 0; pk < kPackets; ++pk) {
            const double *x = term + pk * kX;
            double f;
            if constexpr (kX == 1) f = x[0];
            else if constexpr (kX == 2) f = x[0] + x[1];
            else f = (x[0] + x[1]) + (x[2] + x[3]);
            v[pk] = wave_pair_tree(f);
        }
        if (lane == 0) s_part[which][wave] = kPackets == 1 ? v[0] : v[0] + v[kPackets - 1];
    };
    // wave 0, after a barrier: the sum over the workgroup's blocks
    auto workgroup_sum = [&](int which) -> double {
        return wave_pair_tree(lane < (uint32_t)kParts ? s_part[which][lane] : 0.0);
    };

    // ---- Eq. 1-2 state and Eq. 5
    float alpha1 = alpha0;
    float rho[R];
#pragma unroll
    for (int k = 0; k < R; ++k) rho[k] = 0.0f;
    if constexpr (METHOD == SOAR_METHOD_SOAR) {
        if (!degenerate) {                                   // uniform over the grid
            double tN[R], tM[R];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                tN[k] = tM[k] = 0.0;
                if (blk(k) < t.nblk) {
                    float w[16], q[16];
                    uint32_t nib[2], c0;
                    float delta0, a, b;
                    widen(k, w);
                    block_init(w, alpha0, alpha0_m, c0, delta0, nib, q);
                    block_sums(w, q, a, b);
                    tN[k] = (double)a * (double)delta0;
                    tM[k] = ((double)b * (double)delta0) * (double)delta0;
                    rho[k] = (b == 0.0f) ? -delta0 : a / b;      // first half of Eq. 6
                }
            }
            wave_sum_to_lds(0, tN);
            wave_sum_to_lds(1, tM);
            __syncthreads();
            if (wave == 0) {
                double NM[2] = {workgroup_sum(0), workgroup_sum(1)};
                bool ok = true;
                if (grid.G > 1u) {
                    ok = resident_cross_sums<2>(grid, kResNM1, kResNM2, NM);
                    if (!ok && lane == 0) give_up();
                }
                if (lane == 0) {
                    s_alpha1 = (NM[1] > 0.0) ? (float)(NM[0] / NM[1]) : alpha0;
                    s_gone = ok ? 0u : 1u;
                }
            }
            __syncthreads();
            if (s_gone) return;
            alpha1 = s_alpha1;
        } else if (allzero) {
            alpha1 = 1.0f;
        }
        if (blockIdx.x == 0u && tid == 0) *t.gscale = alpha1;
    }
    const float inv_alpha1 = __builtin_amdgcn_rcpf(alpha1);
    const bool full_search = args.full_search != 0;

    // ---- Eq. 6, new assignment, Eq. 8 search (k_search, per block); the lane's bytes leave together
    double terr[R];
    uint32_t nibs[R][2], codes4 = 0u;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        terr[k] = 0.0;
        nibs[k][0] = nibs[k][1] = 0u;
        if (blk(k) < t.nblk) {
            float w[16], q[16];
            uint32_t out_code;
            float out_err;
            widen(k, w);
            if (allzero) {
                float x[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) x[j] = w[j];
                nibs[k][0] = fp4x8(x);
                nibs[k][1] = fp4x8(x + 8);
                out_code = kE4M3Min;
                out_err = 0.0f;
            } else if constexpr (METHOD == SOAR_METHOD_RTN) {
                uint32_t c0;
                float delta0;
                block_init(w, alpha0, alpha0_m, c0, delta0, nibs[k], q);
                out_code = c0;
                out_err = block_error(w, q, alpha0 * delta0);
            } else {
                const float delta_star = (rho[k] < 0.0f) ? -rho[k] : rho[k] / alpha1;
                const int centre = (int)e4m3_project(delta_star);
                assign_codes(w, alpha1 * delta_star, nibs[k], q);
                int best;
                float best_err;
                bool done = false;
                if (!full_search) {
                    done = search_certified(w, q, alpha1, inv_alpha1, centre, args.radius, best, best_err);
                    if (args.search_stats) count_search(args.search_stats, done);
                }
                if (!done) search_full(w, q, alpha1, centre, args.radius, best, best_err);
                out_code = (uint32_t)best;
                out_err = best_err;
            }
            codes4 |= out_code << (8 * k);
            terr[k] = (double)out_err;
        }
    }
#pragma unroll
    for (int pk = 0; pk < kPackets; ++pk) {
        // streaming stores (the outputs are not read again here).  A packet with all its kX blocks present and
        // the output addresses aligned for it: the 8 kX code bytes in 16-byte pieces, the kX scale bytes in one piece.
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        const uint32_t b0 = blk(pk * kX);
        const bool whole = b0 + (uint32_t)kX <= t.nblk;
        uint8_t *cp = t.codes + (size_t)b0 * 8;
        uint8_t *sp = t.scales + b0;
        const uint32_t (*nb)[2] = nibs + pk * kX;
        const uint32_t sc = codes4 >> (8 * pk * kX);
        if (kX >= 2 && whole && (reinterpret_cast<uintptr_t>(t.codes) & 15u) == 0u) {
#pragma unroll
            for (int k = 0; k < kX; k += 2)
                __builtin_nontemporal_store(u32x4{nb[k][0], nb[k][1], nb[k + (kX >= 2 ? 1 : 0)][0], nb[k + (kX >= 2 ? 1 : 0)][1]},
                                            reinterpret_cast<u32x4 *>(cp) + k / 2);
        } else {
#pragma unroll
            for (int k = 0; k < kX; ++k)
                if (b0 + (uint32_t)k < t.nblk)
                    __builtin_nontemporal_store(u32x2{nb[k][0], nb[k][1]}, reinterpret_cast<u32x2 *>(cp) + k);
        }
        if (kX == 4 && whole && (reinterpret_cast<uintptr_t>(t.scales) & 3u) == 0u) {
            __builtin_nontemporal_store(sc, reinterpret_cast<uint32_t *>(sp));
        } else if (kX == 2 && whole && (reinterpret_cast<uintptr_t>(t.scales) & 1u) == 0u) {
            __builtin_nontemporal_store((uint16_t)sc, reinterpret_cast<uint16_t *>(sp));
        } else {
#pragma unroll
            for (int k = 0; k < kX; ++k)
                if (b0 + (uint32_t)k < t.nblk) __builtin_nontemporal_store((uint8_t)(sc >> (8 * k)), sp + k);
        }
    }
    wave_sum_to_lds(2, terr);
    __syncthreads();
    if (wave != 0) return;
    // ---- error sum and status: workgroup 0 collects
    double total = workgroup_sum(2);
    bool ok = true;
    if (grid.G > 1u) {
        if (t.sse) ok = resident_collect_sum(grid, kResErr1, total);
        if (ok && grid.g != 0u) return;
    }
    if (lane == 0) {
        if (!ok) { give_up(); return; }
        if (t.sse) *t.sse = total;
        if (t.status) *t.status = (amax_bits >= 0x7F800000u ? SOAR_STATUS_NONFINITE : 0) | (allzero ? SOAR_STATUS_ALLZERO : 0);
        if (METHOD == SOAR_METHOD_RTN) *t.gscale = allzero ? 1.0f : alpha0;
    }
}

}  // namespace
