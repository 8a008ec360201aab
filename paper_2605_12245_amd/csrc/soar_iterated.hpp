// The iterated path: Algorithm 1 in full (Sec. 3.3-3.4, Appendix B.3) and the arms of the
// component study: k_iter_init builds the Eq. 1-2 state, k_iter carries out one iteration.
#pragma once
#include "soar_device.hpp"

namespace {

// Sums of up to three per-block binary64 terms over the blocks of a workgroup, as the
// adjacent-pair tree over the flat block index: wave tree, four waves, then a
// binary-counter stack over the workgroup's consecutive tiles.  Call once per tile
// (tile k of the workgroup, all lanes); after the last tile lane 0 holds the sums.
template <int NS>
struct TileTree {
    double (*s_wave)[4];     // [NS][4]
    double (*s_stack)[32];   // [NS][32]
    double wg[NS] = {};
    __device__ __forceinline__ void add_tile(uint32_t k, const double term[NS])
    {
        double v[NS];
#pragma unroll
        for (int n = 0; n < NS; ++n) v[n] = wave_pair_tree(term[n]);
        __syncthreads();                                   // s_wave free again
        if ((threadIdx.x & 63) == 0)
#pragma unroll
            for (int n = 0; n < NS; ++n) s_wave[n][threadIdx.x >> 6] = v[n];
        __syncthreads();
        if (threadIdx.x == 0) {
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                double x = (s_wave[n][0] + s_wave[n][1]) + (s_wave[n][2] + s_wave[n][3]);
                uint32_t lvl = 0;
                while ((k >> lvl) & 1u) { x = s_stack[n][lvl] + x; ++lvl; }
                s_stack[n][lvl] = x;
                wg[n] = x;
            }
        }
    }
};

// The same three sums for the memory-bound kernels, at a fraction of the cross-lane work: what a block
// contributes -- a = sum w q, b = sum q^2, its stored scale d and its error, four floats -- is staged in LDS
// for up to kStage consecutive tiles; lane t then forms the binary64 terms a d, b d^2, err of the adjacent
// blocks t*T .. t*T+T-1 (exact products, wherever they are formed), folds them in registers, and ONE wave
// tree, the four waves and the binary-counter stack finish the group -- the adjacent-pair tree again
// (k_stats does the same for its two sums).  Per group of T tiles: stage() once per tile by every lane,
// then close() by every lane; after the last group lane 0 holds the sums (N, M, error) in wg[].
struct StagedTree {
    float4 *s_blocks;        // [kStage * kWG]: a, b, d, err; zeros for a block that does not exist
    double (*s_wave)[4];     // [3][4]
    double (*s_stack)[32];   // [3][32]
    double wg[3] = {};
    __device__ __forceinline__ void stage(uint32_t kk, float a, float b, float d, float err)
    {
        s_blocks[kk * kWG + threadIdx.x] = make_float4(a, b, d, err);
    }
    static __device__ __forceinline__ void terms(const float4 &x, double v[3])
    {
        v[0] = (double)x.x * (double)x.z;
        v[1] = ((double)x.y * (double)x.z) * (double)x.z;
        v[2] = (double)x.w;
    }
    // group `k` of the workgroup, T tiles staged (T a power of two <= kStage)
    __device__ __forceinline__ void close(uint32_t k, uint32_t T)
    {
        __syncthreads();
        const float4 *x = s_blocks + threadIdx.x * T;
        double v[3];
        terms(x[0], v);
        if (T >= 2) {
            double u[3];
            terms(x[1], u);
#pragma unroll
            for (int n = 0; n < 3; ++n) v[n] = v[n] + u[n];
        }
        if (T == 4) {
            double u[3], z[3];
            terms(x[2], u);
            terms(x[3], z);
#pragma unroll
            for (int n = 0; n < 3; ++n) v[n] = v[n] + (u[n] + z[n]);
        }
#pragma unroll
        for (int n = 0; n < 3; ++n) v[n] = wave_pair_tree(v[n]);
        if ((threadIdx.x & 63) == 0)
#pragma unroll
            for (int n = 0; n < 3; ++n) s_wave[n][threadIdx.x >> 6] = v[n];
        __syncthreads();
        if (threadIdx.x == 0) {
#pragma unroll
            for (int n = 0; n < 3; ++n) {
                double y = (s_wave[n][0] + s_wave[n][1]) + (s_wave[n][2] + s_wave[n][3]);
                uint32_t lvl = 0;
                while ((k >> lvl) & 1u) { y = s_stack[n][lvl] + y; ++lvl; }
                s_stack[n][lvl] = y;
                wg[n] = y;
            }
        }
    }
};
static_assert(kStage == 4, "StagedTree::close folds up to four tiles");

// largest E4M3 code in [0x01, 0x7E] whose value does not exceed y (0x01 if none does)
__device__ __forceinline__ int e4m3_floor_code(float y)
{
    if (!(y > 0.0f)) return (int)kE4M3Min;                  // zero, negative, NaN
    const int normal = (int)(__float_as_uint(y) >> 20) - (120 << 3);
    const int sub = (int)(fminf(y, 1.0f) * 512.0f);
    const int code = (y >= 0x1p-6f) ? normal : sub;
    return min(max(code, (int)kE4M3Min), (int)kE4M3Max);
}

// 1 / s for s > 0 whose biased exponent lies in [1, 252]: the hardware estimate and one fused
// Newton step.  Compared with the correctly rounded division on every binary32 pattern: identical
// over that whole range (the patterns that differ are subnormal inputs and subnormal quotients).
__device__ __forceinline__ float rcp_midrange(float s)
{
    const float y = __builtin_amdgcn_rcpf(s);
    const float e = __builtin_fmaf(-s, y, 1.0f);
    return __builtin_fmaf(e, y, y);
}

// assign_codes with the reciprocal chosen at compile time; nib carries the previous codes in
// (every byte is overwritten) so that no register has to be cleared first
template <bool FAST>
__device__ __forceinline__ void assign_codes_rcp(const float w[16], float scale, uint32_t nib[2], float q[16])
{
    const float r = FAST ? rcp_midrange(scale) : 1.0f / scale;
    float x[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) x[j] = w[j] * r;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t v = nib[h];
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[8 * h + 0], x[8 * h + 1], 1.0f, 0);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[8 * h + 2], x[8 * h + 3], 1.0f, 1);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[8 * h + 4], x[8 * h + 5], 1.0f, 2);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[8 * h + 6], x[8 * h + 7], 1.0f, 3);
        nib[h] = v;
    }
    fp4x8_values(nib[0], q);
    fp4x8_values(nib[1], q + 8);
}

// The joint search of Sec. 3.3 for one block: factors beta ascending, for each the stored-scale
// candidates in their order (bracket: c0 then c0+1; window: c0, -1, +1, ...), the first pair with
// the smallest binary32 error wins.  Only the error and the winning factor are tracked in the
// loop; the winner's codes are formed once more at the end.
template <bool FAST>
__device__ __forceinline__ void joint_search(const float w[16], float alpha, float delta_star, const float *s_beta,
                                             int n_beta, bool bracket, int c0, int radius, float &best_err,
                                             int &best_code, uint32_t best_nib[2], float q[16])
{

    uint32_t nib[2] = {0u, 0u};
    float best = __builtin_inff();           // an error is never NaN; "first wins" for an infinite one too
    float best_beta = s_beta[0];
    if (bracket) {
        const int lo = c0;
        const int hi = min(lo + 1, (int)kE4M3Max);           // hi == lo can never win
        const float s_lo = alpha * e4m3_value((uint32_t)lo);
        const float s_hi = alpha * e4m3_value((uint32_t)hi);
#pragma unroll 4
        for (int kb = 0; kb < n_beta; ++kb) {
            const float bk = s_beta[kb];
            assign_codes_rcp<FAST>(w, alpha * (delta_star * bk), nib, q);
            const float e_lo = block_error(w, q, s_lo);
            const float e_hi = block_error(w, q, s_hi);
            const float m = fminf(fminf(best, e_lo), e_hi);
            best_beta = (m < best) ? bk : best_beta;         // strictly better only: the first factor keeps a tie
            best = m;
        }
        // the winning factor once more: its codes, and which of the two stored scales it won with
        assign_codes_rcp<FAST>(w, alpha * (delta_star * best_beta), best_nib, q);
        const float e_lo = block_error(w, q, s_lo);
        const float e_hi = block_error(w, q, s_hi);
        const bool upper = e_hi < e_lo;                      // the lower code comes first and keeps a tie
        best_code = upper ? hi : lo;
        best_err = upper ? e_hi : e_lo;
    } else {
        best_code = c0;
        for (int kb = 0; kb < n_beta; ++kb) {
            const float bk = s_beta[kb];
            assign_codes_rcp<FAST>(w, alpha * (delta_star * bk), nib, q);
            // a code clamped into [0x01, 0x7E] repeats an earlier candidate of the same factor
            // and can then never win
            for (int c = 0; c <= 2 * radius; ++c) {
                const int o = (c + 1) >> 1;
                const int code = (c & 1) ? max(c0 - o, (int)kE4M3Min) : min(c0 + o, (int)kE4M3Max);
                const float e = block_error(w, q, alpha * e4m3_value((uint32_t)code));
                if (e < best) { best = e; best_beta = bk; best_code = code; }
            }
        }
        best_err = best;
        assign_codes_rcp<FAST>(w, alpha * (delta_star * best_beta), best_nib, q);
    }
}

// assign_codes_rcp without the decoded values (codes only)
template <bool FAST>
__device__ __forceinline__ void codes_only_rcp(const float w[16], float scale, uint32_t nib[2])
{
    const float r = FAST ? rcp_midrange(scale) : 1.0f / scale;
    float x[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) x[j] = w[j] * r;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t v = nib[h];
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[8 * h + 0], x[8 * h + 1], 1.0f, 0);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[8 * h + 2], x[8 * h + 3], 1.0f, 1);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[8 * h + 4], x[8 * h + 5], 1.0f, 2);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[8 * h + 6], x[8 * h + 7], 1.0f, 3);
        nib[h] = v;
    }
}

constexpr int kMaxListBeta = 128;        // longest factor grid the two-pass form of the search handles

// The same joint search in two passes.  Neighbouring factors very often give a block the same 16
// codes (a quarter of the paper's 101 factors give new ones, on average, on heavy-tailed weights),
// and a pair whose codes equal those of the factor before it has the same errors and can never be
// strictly better.  Pass 1 walks all factors, forms the codes only and notes in LDS the factors at
// which this block's codes change; pass 2 evaluates the errors for the noted factors alone (its
// trip count is the longest list in the wave).  The result is that of joint_search, pair for pair.
// list: kMaxListBeta x kWG bytes, entry e of this lane at list[e * kWG + threadIdx.x].
template <bool FAST>
__device__ __forceinline__ void joint_search_two_pass(const float w[16], float alpha, float delta_star,
                                                      const float *s_beta, int n_beta, bool bracket, int c0,
                                                      int radius, uint8_t *list, float &best_err, int &best_code,
                                                      uint32_t best_nib[2], float q[16])
{
    uint32_t nib[2] = {0u, 0u};
    uint32_t p0 = 0u, p1 = 0u;
    int n = 0;
    for (int kb = 0; kb < n_beta; ++kb) {
        codes_only_rcp<FAST>(w, alpha * (delta_star * s_beta[kb]), nib);
        if (kb == 0 || nib[0] != p0 || nib[1] != p1) {
            list[n * kWG + threadIdx.x] = (uint8_t)kb;
            ++n;
        }
        p0 = nib[0];
        p1 = nib[1];
    }
    float best = __builtin_inff();
    float best_beta = s_beta[0];
    const int lo = c0;
    const int hi = min(lo + 1, (int)kE4M3Max);
    const float s_lo = alpha * e4m3_value((uint32_t)lo);
    const float s_hi = alpha * e4m3_value((uint32_t)hi);
    best_code = c0;
    for (int j = 0; __builtin_amdgcn_ballot_w64(j < n) != 0ull; ++j) {
        if (j < n) {
            const float bk = s_beta[list[j * kWG + threadIdx.x]];
            assign_codes_rcp<FAST>(w, alpha * (delta_star * bk), nib, q);
            if (bracket) {
                const float e_lo = block_error(w, q, s_lo);
                const float e_hi = block_error(w, q, s_hi);
                const float m = fminf(fminf(best, e_lo), e_hi);
                best_beta = (m < best) ? bk : best_beta;
                best = m;
            } else {
                for (int c = 0; c <= 2 * radius; ++c) {
                    const int o = (c + 1) >> 1;
                    const int code = (c & 1) ? max(c0 - o, (int)kE4M3Min) : min(c0 + o, (int)kE4M3Max);
                    const float e = block_error(w, q, alpha * e4m3_value((uint32_t)code));
                    if (e < best) { best = e; best_beta = bk; best_code = code; }
                }
            }
        }
    }
    assign_codes_rcp<FAST>(w, alpha * (delta_star * best_beta), best_nib, q);
    if (bracket) {
        const float e_lo = block_error(w, q, s_lo);
        const float e_hi = block_error(w, q, s_hi);
        const bool upper = e_hi < e_lo;
        best_code = upper ? hi : lo;
        best_err = upper ? e_hi : e_lo;
    } else {
        best_err = best;
    }
}

// The Eq. 1-2 state of Algorithm 1 (Delta^q = Delta^d = Delta0) for the iterated
// path: per block the ratio a/b for Eq. 6 and the error of that state; per tensor
// the sums of Eq. 5 (-> the global scale of iteration 0) and the error before any
// iteration.
template <int DT>
__global__ __launch_bounds__(kWG) void k_iter_init(const Batch batch)
{
    __shared__ float4 s_blocks[kStage * kWG];
    __shared__ double s_wave[3][4];
    __shared__ double s_stack[3][32];
    __shared__ uint32_t s_last;
    double *s_tree = reinterpret_cast<double *>(s_blocks);      // trees_of_partials, after the last group
    static_assert(sizeof(float4) * kStage >= sizeof(double), "s_tree fits s_blocks");

    uint32_t lwg;
    const Task t = batch.t[find_task(batch, lwg)];
    const uint32_t tid = threadIdx.x;
    const uint32_t amax_bits = t.ctrl->amax_bits;
    const bool degenerate = amax_bits == 0u || amax_bits >= 0x7F800000u;
    const float alpha0 = f_of(amax_bits) / 2688.0f;
    const float alpha0_m = alpha0 * 6.0f;

    StagedTree tree{s_blocks, s_wave, s_stack};
    const uint32_t tile0 = lwg * t.tiles_per_wg;
    const uint32_t T = t.tiles_per_wg < (uint32_t)kStage ? t.tiles_per_wg : (uint32_t)kStage;   // power of two
    for (uint32_t kg = 0; kg < t.tiles_per_wg; kg += T) {
        for (uint32_t kk = 0; kk < T; ++kk) {
            const uint32_t i = (tile0 + kg + kk) * kWG + tid;
            float a = 0.0f, b = 0.0f, delta0 = 0.0f, err = 0.0f;
            if (i < t.nblk) {
                float rho = 0.0f;
                if (!degenerate) {
                    float w[16], q[16];
                    uint32_t nib[2], c0;
                    load_block<DT>(t.w, block_offset(t, i), w);
                    block_init(w, alpha0, alpha0_m, c0, delta0, nib, q);
                    block_sums(w, q, a, b);
                    err = block_error(w, q, alpha0 * delta0);
                    rho = (b == 0.0f || batch.arm == SOAR_METHOD_DSS_ONLY) ? -delta0 : a / b;
                }
                t.rho[i] = rho;
            }
            tree.stage(kk, a, b, delta0, err);
        }
        tree.close(kg / T, T);
    }
    uint32_t *counters = t.counters + 1 * kSlots * kSlotStride;
    if (tid == 0) {
        publish(t.part + lwg, tree.wg[0]);
        publish(t.part + kMaxPartials + lwg, tree.wg[1]);
        publish(t.part + 2 * kMaxPartials + lwg, tree.wg[2]);
        s_last = arrive_is_last(counters, &t.ctrl->top[1], t.n_wg, lwg) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    double NME[3];
    trees_of_partials<3>(t.part, t.n_wg, s_tree, &s_stack[0][0], NME);
    const double N = NME[0], M = NME[1], E = NME[2];
    if (tid == 0) {
        t.ctrl->alpha0 = alpha0;
        // the global scale of iteration 0: Eq. 5, or unchanged when the closed-form stage is left out
        t.ctrl->alpha1 = (M > 0.0 && batch.arm != SOAR_METHOD_DSS_ONLY) ? (float)(N / M) : alpha0;
        t.ctrl->N = N;
        t.ctrl->M = M;
        t.ctrl->prev_sse = E;
        t.ctrl->stopped = 0u;
        if (!degenerate && t.trace) t.trace[0] = E;
    }
    reset_counters(counters, &t.ctrl->top[1]);
}

// What the last workgroup of a tensor does after an iteration (one lane): the outputs that describe the
// tensor, the early-stop decision and the global scale the next iteration starts from (Eq. 5).
__device__ __forceinline__ void finish_iteration(const Batch &batch, const Task &t, double N, double M, double cur, float alpha,
                                                 bool degenerate, bool allzero, bool dss_only)
{
    if (degenerate) {
        *t.gscale = allzero ? 1.0f : __builtin_nanf("");
        if (t.sse) *t.sse = allzero ? 0.0 : __builtin_nan("");
        if (t.status) *t.status = allzero ? SOAR_STATUS_ALLZERO : SOAR_STATUS_NONFINITE;
        if (t.iters_run) *t.iters_run = 0;
    } else {
        const double prev = t.ctrl->prev_sse;
        *t.gscale = alpha;
        if (t.sse) *t.sse = cur;
        if (t.status) *t.status = 0;
        if (t.iters_run) *t.iters_run = batch.iter_t + 1;
        if (t.trace) t.trace[batch.iter_t + 1] = cur;
        const bool stop = batch.early_stop_rel > 0.0f && (prev - cur) < (double)batch.early_stop_rel * prev;
        t.ctrl->stopped = stop ? 1u : 0u;
        t.ctrl->prev_sse = cur;
        t.ctrl->alpha1 = (M > 0.0 && !dss_only) ? (float)(N / M) : alpha;      // Eq. 5 for the next iteration
        t.ctrl->N = N;
        t.ctrl->M = M;
    }
}

// One iteration of Algorithm 1.  On entry ctrl->alpha1 holds the Eq. 5 global
// scale for the current codes and stored scales and rho[i] the block ratio a/b
// (Eq. 6 is rho / alpha).  Per block: the joint search of Sec. 3.3 over
// (factor beta ascending) x (stored-scale candidates in their order), keeping
// the first pair with the smallest binary32 error; the block's codes, stored
// scale, and -- because the codes of the winning pair ARE the codes the next
// iteration starts from -- the next a/b and Eq. 5 terms.  Per tensor: the error
// after this iteration (exact adjacent-pair tree, so that the early-stop test
// is reproducible), the stop flag and the next global scale.
// A tensor whose stop flag is set is skipped by every later launch.
template <int DT>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(4, 8))) void k_iter(const Batch batch)
{
    __shared__ double s_wave[3][4];
    __shared__ double s_stack[3][32];
    __shared__ double s_tree[kWG];
    // dynamic LDS: the factor table (n_beta floats, rounded up to 256 bytes), then, for the two-pass
    // search, the change lists (n_beta x kWG bytes)
    extern __shared__ __align__(16) unsigned char s_dyn[];
    float *s_beta = reinterpret_cast<float *>(s_dyn);
    uint8_t *s_list = s_dyn + ((size_t)batch.n_beta * 4 + 255) / 256 * 256;
    __shared__ uint32_t s_last;

    uint32_t lwg;
    const Task t = batch.t[find_task(batch, lwg)];
    const uint32_t tid = threadIdx.x;
    const uint32_t amax_bits = t.ctrl->amax_bits;
    const bool allzero = amax_bits == 0u;
    const bool degenerate = allzero || amax_bits >= 0x7F800000u;
    if (degenerate ? batch.iter_t != 0 : t.ctrl->stopped != 0u) return;     // uniform over the tensor's workgroups

    const int n_beta = batch.n_beta;
    for (int k = (int)tid; k < n_beta; k += kWG)
        s_beta[k] = n_beta <= 1 ? batch.beta_lo
                                : (batch.beta_lo * (float)(n_beta - 1 - k) + batch.beta_hi * (float)k) / (float)(n_beta - 1);
    __syncthreads();

    const float alpha = t.ctrl->alpha1;
    const bool bracket = batch.dd_mode == SOAR_DD_BRACKET;
    const int radius = batch.radius;
    const bool two_pass = n_beta >= 4 && n_beta <= kMaxListBeta && !batch.full_search;
    const bool dss_only = batch.arm == SOAR_METHOD_DSS_ONLY;    // rho then always carries -Delta^d: the search centre

    TileTree<3> tree{s_wave, s_stack};
    const uint32_t tile0 = lwg * t.tiles_per_wg;
    for (uint32_t k = 0; k < t.tiles_per_wg; ++k) {
        const uint32_t i = (tile0 + k) * kWG + tid;
        double term[3] = {0.0, 0.0, 0.0};
        if (i < t.nblk && amax_bits < 0x7F800000u) {
            float w[16], q[16];
            uint32_t best_nib[2] = {0u, 0u};
            int best_code = (int)kE4M3Min;
            float best_err = 0.0f;
            load_block<DT>(t.w, block_offset(t, i), w);
            if (allzero) {
                float x[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) x[j] = w[j];
                best_nib[0] = fp4x8(x);
                best_nib[1] = fp4x8(x + 8);
            } else {
                const float rho = t.rho[i];
                const float delta_star = (rho < 0.0f) ? -rho : rho / alpha;
                const int c0 = bracket ? e4m3_floor_code(delta_star) : (int)e4m3_project(delta_star);
                // the reciprocal shortcut holds while the biased exponent of the scale stays in [1, 252];
                // the scales of a block lie between those of the first and the last factor (to within
                // rounding of the grid), which are asked to keep one binade of distance from both ends
                const float s_first = alpha * (delta_star * s_beta[0]);
                const float s_final = alpha * (delta_star * s_beta[n_beta - 1]);
                const bool mid = ((__float_as_uint(s_first) >> 23) - 2u) < 250u && ((__float_as_uint(s_final) >> 23) - 2u) < 250u;
                if (two_pass) {
                    if (__builtin_amdgcn_ballot_w64(!mid) == 0ull)
                        joint_search_two_pass<true>(w, alpha, delta_star, s_beta, n_beta, bracket, c0, radius, s_list,
                                                    best_err, best_code, best_nib, q);
                    else
                        joint_search_two_pass<false>(w, alpha, delta_star, s_beta, n_beta, bracket, c0, radius, s_list,
                                                     best_err, best_code, best_nib, q);
                } else if (__builtin_amdgcn_ballot_w64(!mid) == 0ull) {
                    joint_search<true>(w, alpha, delta_star, s_beta, n_beta, bracket, c0, radius, best_err, best_code,
                                       best_nib, q);
                } else {
                    joint_search<false>(w, alpha, delta_star, s_beta, n_beta, bracket, c0, radius, best_err, best_code,
                                        best_nib, q);
                }
                // the state the next iteration starts from
                float a, b;
                block_sums(w, q, a, b);
                const float d = e4m3_value((uint32_t)best_code);
                term[0] = (double)a * (double)d;
                term[1] = ((double)b * (double)d) * (double)d;
                term[2] = (double)best_err;
                t.rho[i] = (b == 0.0f || dss_only) ? -d : a / b;
            }
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            u32x2 packed = {best_nib[0], best_nib[1]};
            reinterpret_cast<u32x2 *>(t.codes)[i] = packed;
            t.scales[i] = (uint8_t)best_code;
        }
        tree.add_tile(k, term);
    }
    uint32_t *counters = t.counters + 2 * kSlots * kSlotStride;
    if (tid == 0) {
        publish(t.part + lwg, tree.wg[0]);
        publish(t.part + kMaxPartials + lwg, tree.wg[1]);
        publish(t.part + 2 * kMaxPartials + lwg, tree.wg[2]);
        s_last = arrive_is_last(counters, &t.ctrl->top[2], t.n_wg, lwg) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    double NME[3];
    trees_of_partials<3>(t.part, t.n_wg, s_tree, &s_stack[0][0], NME);
    const double N = NME[0], M = NME[1], cur = NME[2];
    if (tid == 0) finish_iteration(batch, t, N, M, cur, alpha, degenerate, allzero, dss_only);
    reset_counters(counters, &t.ctrl->top[2]);
}

// One iteration of the closed-form arm of the component study (Sec. 3.2 alone): no search.  Per block the
// projected scale E4M3(Delta*) assigns the codes AND is stored; the codes' a/b and Eq. 5 terms are formed
// for the next iteration as in k_iter, and the tensor is finished by finish_iteration.  The kernel is bound
// by memory (weights and ratio read, ratio, codes and scale written), so it is built like k_stats: several
// consecutive tiles per workgroup, the three sums through the staged tree, streaming stores for the outputs
// (the weights and the ratio are read again by the next iteration and stay in the last-level cache).
// (held to 64 registers: eight waves per SIMD hide the loads of this memory-bound kernel)
template <int DT>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(8))) void k_cjso(const Batch batch)
{
    __shared__ float4 s_blocks[kStage * kWG];
    __shared__ double s_wave[3][4];
    __shared__ double s_stack[3][32];
    __shared__ uint32_t s_last;
    double *s_tree = reinterpret_cast<double *>(s_blocks);      // trees_of_partials, after the last group

    uint32_t lwg;
    const Task t = batch.t[find_task(batch, lwg)];
    const uint32_t tid = threadIdx.x;
    const uint32_t amax_bits = t.ctrl->amax_bits;
    const bool allzero = amax_bits == 0u;
    const bool degenerate = allzero || amax_bits >= 0x7F800000u;
    if (degenerate ? batch.iter_t != 0 : t.ctrl->stopped != 0u) return;     // uniform over the tensor's workgroups
    const float alpha = t.ctrl->alpha1;

    StagedTree tree{s_blocks, s_wave, s_stack};
    const uint32_t tile0 = lwg * t.tiles_per_wg;
    const uint32_t T = t.tiles_per_wg < (uint32_t)kStage ? t.tiles_per_wg : (uint32_t)kStage;   // power of two
    for (uint32_t kg = 0; kg < t.tiles_per_wg; kg += T) {
        for (uint32_t kk = 0; kk < T; ++kk) {
            const uint32_t i = (tile0 + kg + kk) * kWG + tid;
            float a = 0.0f, b = 0.0f, d = 0.0f, err = 0.0f;
            if (i < t.nblk && amax_bits < 0x7F800000u) {
                float w[16], q[16];
                uint32_t nib[2] = {0u, 0u};
                uint32_t code = kE4M3Min;
                load_block<DT>(t.w, block_offset(t, i), w);
                if (allzero) {
                    float x[16];
#pragma unroll
                    for (int j = 0; j < 16; ++j) x[j] = w[j];
                    nib[0] = fp4x8(x);
                    nib[1] = fp4x8(x + 8);
                } else {
                    const float rho = t.rho[i];
                    const float delta_star = (rho < 0.0f) ? -rho : rho / alpha;          // Eq. 6
                    code = e4m3_project(delta_star);
                    d = e4m3_value(code);
                    const float sd = alpha * d;
                    assign_codes(w, sd, nib, q);
                    block_sums(w, q, a, b);
                    err = block_error(w, q, sd);
                    t.rho[i] = (b == 0.0f) ? -d : a / b;
                }
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                u32x2 packed = {nib[0], nib[1]};
                __builtin_nontemporal_store(packed, reinterpret_cast<u32x2 *>(t.codes) + i);
                __builtin_nontemporal_store((uint8_t)code, t.scales + i);
            }
            tree.stage(kk, a, b, d, err);
        }
        tree.close(kg / T, T);
    }
    uint32_t *counters = t.counters + 2 * kSlots * kSlotStride;
    if (tid == 0) {
        publish(t.part + lwg, tree.wg[0]);
        publish(t.part + kMaxPartials + lwg, tree.wg[1]);
        publish(t.part + 2 * kMaxPartials + lwg, tree.wg[2]);
        s_last = arrive_is_last(counters, &t.ctrl->top[2], t.n_wg, lwg) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    double NME[3];
    trees_of_partials<3>(t.part, t.n_wg, s_tree, &s_stack[0][0], NME);
    const double N = NME[0], M = NME[1], cur = NME[2];
    if (tid == 0) finish_iteration(batch, t, N, M, cur, alpha, degenerate, allzero, false);
    reset_counters(counters, &t.ctrl->top[2]);
}

}  // namespace
