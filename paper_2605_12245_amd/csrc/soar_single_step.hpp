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
    const Task t = batch.t[find_task(batch, lwg)];
    const uint32_t tid = threadIdx.x;
    constexpr int kChunks = DT == SOAR_BF16 ? 2 : 4;      // 16-byte pieces per block

    // tiles are dealt round-robin over the tensor's workgroups, so that at any moment
    // the workgroups in flight sweep one contiguous window of memory
    uint32_t m = 0;
    for (uint32_t k = 0; k < t.tiles_per_wg; ++k) {
        const uint32_t i = (k * t.n_wg + lwg) * kWG + tid;
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
        const uint32_t ns = t.n_wg < (uint32_t)kSlots ? t.n_wg : (uint32_t)kSlots;
        // arrive_is_last waits for this read-modify-write to complete before it counts the workgroup in
        __hip_atomic_fetch_max(t.slot_max + (lwg % ns) * kSlotStride, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = arrive_is_last(counters, &t.ctrl->top[0], t.n_wg, lwg) ? 1u : 0u;
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
    const double N = tree_of_partials(partN, t.n_wg, s_tree, s_stack[0]);
    const double M = tree_of_partials(partM, t.n_wg, s_tree, s_stack[1]);
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
    const bool margin_ok = best_err < 512.0f * (C * (sa * sa));
    const bool range_ok = (B > 0x1p-100f) && (best_err > 0x1p-100f) && (C > 0.0f);
    return left_ok && right_ok && margin_ok && range_ok;
}

// Eq. 6, projection, new assignment, Eq. 8 search, packing, error sum.
// METHOD RTN emits the Eq. 1-2 state instead.
template <int DT, int METHOD>
__global__ __launch_bounds__(kWG) void k_search(const Batch batch)
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
    const Task t = batch.t[find_task(batch, lwg)];
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
    for (uint32_t k = 0; k < t.tiles_per_wg; ++k) {
        const uint32_t i = (k * t.n_wg + lwg) * kWG + tid;
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
            if (!full_search) done = search_certified(w, q, alpha1, inv_alpha1, centre, radius, best, best_err);
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
        s_last = arrive_is_last(counters, &t.ctrl->top[2], t.n_wg, lwg) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    const double total = tree_of_partials(partS, t.n_wg, s_tree, s_stack);
    if (tid == 0) {
        if (t.sse) *t.sse = total;
        if (t.status)
            *t.status = bad_amax ? SOAR_STATUS_BAD_AMAX
                                 : (amax_bits >= 0x7F800000u ? SOAR_STATUS_NONFINITE : 0) | (allzero ? SOAR_STATUS_ALLZERO : 0);
        if (METHOD == SOAR_METHOD_RTN) *t.gscale = allzero ? 1.0f : alpha0;
    }
    reset_counters(counters, &t.ctrl->top[2]);
}

// The whole single-step path for one small tensor in one workgroup: a tensor of at most
// kSmallBlocks blocks is latency-bound on the four dependent launches of the path above; here the
// 1024 lanes keep their (up to four) blocks in registers, and the two tensor-wide results cross
// the workgroup through LDS and a barrier.  Same arithmetic, same trees: lane `tid` owns the
// blocks tid, tid + 1024, ...; a wave's DPP tree sums 64 consecutive blocks, and the 4 x 16 wave
// sums, laid out in block order over the lanes of wave 0, go through the same DPP tree again --
// together the adjacent-pair tree over the flat block index, zero-padded.  No workspace is used.
constexpr int kSmallWG = 1024;
constexpr int kSmallPer = 4;                               // blocks per lane, at most
constexpr uint32_t kSmallBlocks = kSmallWG * kSmallPer;
template <int DT, int METHOD>
__global__ __launch_bounds__(kSmallWG) void k_small(const Task t, const int radius, const int full_search)
{
    constexpr int kWaves = kSmallWG / 64;
    constexpr int kP = pieces_per_block<DT, 16>();
    __shared__ uint32_t s_max[kWaves];
    __shared__ double s_part[3][kSmallPer * kWaves];
    __shared__ float s_alpha1;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;

    // ---- the blocks of this lane, as loaded; Eq. 1 maximum
    u32x4 raw[kSmallPer][kP];
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < kSmallPer; ++k) {
        const uint32_t i = (uint32_t)k * kSmallWG + tid;
#pragma unroll
        for (int p = 0; p < kP; ++p) raw[k][p] = u32x4{0u, 0u, 0u, 0u};
        if (i < t.nblk) {
            const char *src = static_cast<const char *>(t.w) + block_offset(t, i) * (DT == SOAR_BF16 ? 2 : 4);
#pragma unroll
            for (int p = 0; p < kP; ++p) {
                raw[k][p] = load16<false>(src + 16 * p);
                m = absmax_accumulate<DT>(m, make_uint4(raw[k][p].x, raw[k][p].y, raw[k][p].z, raw[k][p].w));
            }
        }
    }
    if constexpr (DT == SOAR_BF16) m = max(m & 0xFFFFu, m >> 16) << 16;
    m = wave_max_u32(m);
    if (lane == 0) s_max[wave] = m;
    __syncthreads();
    uint32_t amax_bits = 0;
#pragma unroll
    for (int w2 = 0; w2 < kWaves; ++w2) amax_bits = max(amax_bits, s_max[w2]);
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
    // sum of one binary64 term per block over the tensor: every lane of the workgroup calls it
    auto tensor_sum = [&](int which, const double term[kSmallPer]) -> double {
#pragma unroll
        for (int k = 0; k < kSmallPer; ++k) {
            const double v = wave_pair_tree(term[k]);
            if (lane == 0) s_part[which][k * kWaves + wave] = v;
        }
        __syncthreads();
        return wave_pair_tree(s_part[which][lane]);        // 4 x 16 wave sums in block order
    };

    // ---- Eq. 1-2 state and Eq. 5
    float alpha1 = alpha0;
    float rho[kSmallPer];
#pragma unroll
    for (int k = 0; k < kSmallPer; ++k) rho[k] = 0.0f;
    if constexpr (METHOD == SOAR_METHOD_SOAR) {
        double tN[kSmallPer], tM[kSmallPer];
#pragma unroll
        for (int k = 0; k < kSmallPer; ++k) {
            tN[k] = tM[k] = 0.0;
            const uint32_t i = (uint32_t)k * kSmallWG + tid;
            if (i < t.nblk && !degenerate) {
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
        const double N = tensor_sum(0, tN);
        const double M = tensor_sum(1, tM);
        if (tid == 0) {
            float a1 = (M > 0.0) ? (float)(N / M) : alpha0;
            if (allzero) a1 = 1.0f;
            s_alpha1 = a1;
            *t.gscale = a1;
        }
        __syncthreads();
        alpha1 = s_alpha1;
    }
    const float inv_alpha1 = __builtin_amdgcn_rcpf(alpha1);

    // ---- Eq. 6, new assignment, Eq. 8 search, packing (k_search, per block)
    double terr[kSmallPer];
#pragma unroll
    for (int k = 0; k < kSmallPer; ++k) {
        terr[k] = 0.0;
        const uint32_t i = (uint32_t)k * kSmallWG + tid;
        if (i < t.nblk) {
            float w[16], q[16];
            uint32_t nib[2], out_code;
            float out_err;
            widen(k, w);
            if (allzero) {
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
                const float delta_star = (rho[k] < 0.0f) ? -rho[k] : rho[k] / alpha1;
                const int centre = (int)e4m3_project(delta_star);
                assign_codes(w, alpha1 * delta_star, nib, q);
                int best;
                float best_err;
                bool done = false;
                if (!full_search) done = search_certified(w, q, alpha1, inv_alpha1, centre, radius, best, best_err);
                if (!done) search_full(w, q, alpha1, centre, radius, best, best_err);
                out_code = (uint32_t)best;
                out_err = best_err;
            }
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            u32x2 packed = {nib[0], nib[1]};
            reinterpret_cast<u32x2 *>(t.codes)[i] = packed;
            t.scales[i] = (uint8_t)out_code;
            terr[k] = (double)out_err;
        }
    }
    const double total = tensor_sum(2, terr);
    if (tid == 0) {
        if (t.sse) *t.sse = total;
        if (t.status) *t.status = (amax_bits >= 0x7F800000u ? SOAR_STATUS_NONFINITE : 0) | (allzero ? SOAR_STATUS_ALLZERO : 0);
        if (METHOD == SOAR_METHOD_RTN) *t.gscale = allzero ? 1.0f : alpha0;
    }
}

}  // namespace
