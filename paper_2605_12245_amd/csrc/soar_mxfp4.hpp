// MXFP4 (blocks of 32, E8M0 scale; OCP Microscaling Formats v1.0), plain conversion or with the
// decoupled scale search of Sec. 3.3 carried over to it (Sec. 4.3): k_mx.
#pragma once
#include "soar_device.hpp"
#include "soar_iterated.hpp"      // TileTree, rcp_midrange

namespace {

// Blocks of 32 elements with an E8M0 scale byte (OCP Microscaling Formats v1.0), plain
// conversion or with the decoupled scale search of Sec. 3.3 carried over to it (Sec. 4.3,
// "DSS on MXFP4").  One lane owns one block of 64 (bf16) or 128 (fp32) bytes.
// There is no tensor-wide scale, so this is a single pass; the only tensor-wide result is the
// error sum (exact adjacent-pair tree, as in the iterated path).
struct MxTask {
    const void *w;
    uint8_t  *codes, *scales;
    double   *sse;
    int32_t  *status;
    int64_t  ld;
    uint32_t bpr;            // 32-element blocks per row
    uint32_t nblk;
    uint32_t tiles_per_wg;
    uint32_t contiguous;
    uint32_t wg_begin;       // first workgroup of the grid that works on this tensor
    uint32_t n_wg;
    Ctrl     *ctrl;          // amax_bits is used as the "saw a non-finite value" flag
    uint32_t *counters;
    double   *part;
    int32_t  dss, n_beta, radius;
    int32_t  two_pass;       // search: codes of every factor first, errors only where they change
    float    beta_lo, beta_hi;
};

struct MxBatch {
    MxTask   t[kGroupMax];
    uint32_t n;
};

// 2^(e-127) for an E8M0 code e in [0, 254]; e = 0 is the binary32 subnormal 2^-127
__device__ __forceinline__ float e8m0_value(int e) { return f_of(e > 0 ? (uint32_t)e << 23 : 0x00400000u); }

template <bool FAST>
__device__ __forceinline__ void mx_assign(const float w[32], float scale, uint32_t nib[4], float q[32])
{
    const float r = FAST ? rcp_midrange(scale) : 1.0f / scale;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = w[8 * h + j] * r;
        uint32_t v = nib[h];
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[0], x[1], 1.0f, 0);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[2], x[3], 1.0f, 1);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[4], x[5], 1.0f, 2);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[6], x[7], 1.0f, 3);
        nib[h] = v;
        fp4x8_values(v, q + 8 * h);
    }
}

// Eq. 8 with alpha = 1 over the 32 elements: one ascending chain of fused operations
__device__ __forceinline__ float mx_block_error(const float w[32], const float q[32], float s)
{
    const float ns = -s;
    float err = 0.0f;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        float e = __builtin_fmaf(q[j], ns, w[j]);
        err = __builtin_fmaf(e, e, err);
    }
    return err;
}

// candidate number c of the search order 0,-1,+1,-2,...; a code outside [0, 254] is clamped onto an
// already evaluated candidate of the same factor and can then never win
__device__ __forceinline__ int mx_candidate(int e0, int c)
{
    const int o = (c + 1) >> 1;
    return (c & 1) ? max(e0 - o, 0) : min(e0 + o, 254);
}

// Least Eq. 8 error over the stored codes e0-K..e0+K for fixed element codes q.  For fixed codes the
// exact error is a parabola in the scale, f(x) = A - 2Bx + Cx^2 with B = sum w q, C = sum q^2 and
// minimiser x* = B/C, and f(2x) < f(x) exactly when x* > 1.5 x: the power of two nearest to x* in
// that sense, clamped to the window, is the winner, and only its error chain is evaluated -- provided
// that x* stays clear of the two decision points next to it by a margin far above the rounding error
// of the computed B/C, and that the exact rise to either neighbour, C x |3x - 2x*|, exceeds the
// worst-case rounding error of the binary32 chains (34 ulp relative, all terms non-negative) by a
// wide factor; candidates further out lie higher still (the bound grows with the rise).  Where that
// cannot be shown for some lane of the wave, the other candidates are evaluated too, as the definition
// says: the result never depends on the shortcut.
__device__ __forceinline__ float mx_window_min(const float w[32], const float q[32], int e0, int radius)
{
    bool sure = false;
    float m = 0.0f;
    int cw = e0;
    {
        float B = 0.0f, C = 0.0f;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            B = __builtin_fmaf(w[j], q[j], B);
            C = __builtin_fmaf(q[j], q[j], C);
        }
        const int lo = max(e0 - radius, 0), hi = min(e0 + radius, 254);
        const float xstar = B * __builtin_amdgcn_rcpf(C);
        // 0.75 * 2^(c-127) < x* <= 1.5 * 2^(c-127)  <=>  c = biased exponent of x* * 4/3 (approximately: checked below)
        cw = (int)(__float_as_uint(xstar * 1.33333337f) >> 23);
        cw = min(max(cw, lo), hi);
        const float xw = e8m0_value(cw);
        m = mx_block_error(w, q, xw);
        // magnitudes at which squares underflow, or overflow, are left to the full evaluation
        sure = C > 0.0f && B > 0x1p-100f && m > 0x1p-100f && m < 0x1p100f && xstar < 0x1p100f && cw >= 2 && cw <= 252;
        const float clear = 0x1p-14f * xstar;       // the computed x* is within 2^-18.8 of the exact one
        if (cw > lo) {
            const float x = 0.5f * xw;
            const float g = 2.0f * xstar - 3.0f * x;
            const float rise = C * x * g;
            sure = sure && g > clear && 0.8f * rise > 0x1p-16f * (m + rise);
        }
        if (cw < hi) {
            const float g = 3.0f * xw - 2.0f * xstar;
            const float rise = C * xw * g;
            sure = sure && g > clear && 0.8f * rise > 0x1p-16f * (m + rise);
        }
    }
    if (__builtin_amdgcn_ballot_w64(!sure) != 0ull) {
        // the 2K other codes of the window (cw is one of them; a code clamped onto [0, 254] repeats another)
        for (int t = 0; t < 2 * radius; ++t) {
            int c = e0 - radius + t;
            c += c >= cw ? 1 : 0;
            m = fminf(m, mx_block_error(w, q, e8m0_value(min(max(c, 0), 254))));
        }
    }
    return m;
}

template <bool FAST>
__device__ __forceinline__ void mx_search(const float w[32], int e0, const float *s_beta, int n_beta, int radius,
                                          float &best_err, int &best_code, uint32_t best_nib[4], float q[32])
{
    const float x0 = e8m0_value(e0);
    uint32_t nib[4] = {0u, 0u, 0u, 0u};
    float best = __builtin_inff();
    float best_beta = s_beta[0];
    for (int kb = 0; kb < n_beta; ++kb) {
        const float bk = s_beta[kb];
        mx_assign<FAST>(w, x0 * bk, nib, q);
        const float m = mx_window_min(w, q, e0, radius);
        best_beta = (m < best) ? bk : best_beta;             // strictly better only: the first factor keeps a tie
        best = fminf(best, m);
    }
    // the winning factor once more: its codes, and the first stored code that reaches its least error
    best_nib[0] = best_nib[1] = best_nib[2] = best_nib[3] = 0u;
    mx_assign<FAST>(w, x0 * best_beta, best_nib, q);
    best_code = e0;
    best_err = mx_block_error(w, q, x0);
    for (int c = 1; c <= 2 * radius; ++c) {
        const int code = mx_candidate(e0, c);
        const float e = mx_block_error(w, q, e8m0_value(code));
        if (e < best_err) { best_err = e; best_code = code; }
    }
}

template <bool FAST>
__device__ __forceinline__ void mx_codes_only(const float w[32], float scale, uint32_t nib[4])
{
    const float r = FAST ? rcp_midrange(scale) : 1.0f / scale;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = w[8 * h + j] * r;
        uint32_t v = nib[h];
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[0], x[1], 1.0f, 0);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[2], x[3], 1.0f, 1);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[4], x[5], 1.0f, 2);
        v = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(v, x[6], x[7], 1.0f, 3);
        nib[h] = v;
    }
}

// mx_search in two passes, as joint_search_two_pass: codes of every factor first, errors only for the
// factors at which this block's codes change (list: n_beta x kWG bytes of LDS)
template <bool FAST>
__device__ __forceinline__ void mx_search_two_pass(const float w[32], int e0, const float *s_beta, int n_beta,
                                                   int radius, uint8_t *list, float &best_err, int &best_code,
                                                   uint32_t best_nib[4], float q[32])
{
    const float x0 = e8m0_value(e0);
    uint32_t nib[4] = {0u, 0u, 0u, 0u};
    uint32_t p[4] = {0u, 0u, 0u, 0u};
    int n = 0;
    for (int kb = 0; kb < n_beta; ++kb) {
        mx_codes_only<FAST>(w, x0 * s_beta[kb], nib);
        if (kb == 0 || nib[0] != p[0] || nib[1] != p[1] || nib[2] != p[2] || nib[3] != p[3]) {
            list[n * kWG + threadIdx.x] = (uint8_t)kb;
            ++n;
        }
#pragma unroll
        for (int h = 0; h < 4; ++h) p[h] = nib[h];
    }
    float best = __builtin_inff();
    float best_beta = s_beta[0];
    for (int j = 0; __builtin_amdgcn_ballot_w64(j < n) != 0ull; ++j) {
        if (j < n) {
            const float bk = s_beta[list[j * kWG + threadIdx.x]];
            mx_assign<FAST>(w, x0 * bk, nib, q);
            const float m = mx_window_min(w, q, e0, radius);
            best_beta = (m < best) ? bk : best_beta;
            best = fminf(best, m);
        }
    }
    best_nib[0] = best_nib[1] = best_nib[2] = best_nib[3] = 0u;
    mx_assign<FAST>(w, x0 * best_beta, best_nib, q);
    best_code = e0;
    best_err = mx_block_error(w, q, x0);
    for (int c = 1; c <= 2 * radius; ++c) {
        const int code = mx_candidate(e0, c);
        const float e = mx_block_error(w, q, e8m0_value(code));
        if (e < best_err) { best_err = e; best_code = code; }
    }
}

template <int DT, bool DSS>
__global__ __launch_bounds__(kWG) void k_mx(const MxBatch batch)
{
    __shared__ double s_wave[1][4];
    __shared__ double s_stack[1][32];
    __shared__ double s_tree[kWG];
    __shared__ uint32_t s_last;
    constexpr int kP = pieces_per_block<DT, 32>();
    __shared__ u32x4 s_x[(DSS || DT != SOAR_BF16) ? 1 : kWG * kP];   // load_wave_blocks: one region per wave
    // dynamic LDS: the factor table (rounded up to 256 bytes), then the change lists of the two-pass search
    extern __shared__ __align__(16) unsigned char s_dyn_mx[];
    float *s_beta = reinterpret_cast<float *>(s_dyn_mx);
    uint8_t *s_list = s_dyn_mx + ((size_t)batch.t[0].n_beta * 4 + 255) / 256 * 256;

    const uint32_t tid = threadIdx.x;
    uint32_t which = 0;
    for (uint32_t j = 1; j < batch.n; ++j)
        if (blockIdx.x >= batch.t[j].wg_begin) which = j;
    const MxTask t = batch.t[which];
    const uint32_t lwg = blockIdx.x - t.wg_begin;
    const int n_beta = DSS ? t.n_beta : 0;
    for (int k = (int)tid; k < n_beta; k += kWG)
        s_beta[k] = n_beta <= 1 ? t.beta_lo
                                : (t.beta_lo * (float)(n_beta - 1 - k) + t.beta_hi * (float)k) / (float)(n_beta - 1);
    __syncthreads();

    TileTree<1> tree{s_wave, s_stack};
    bool nonfinite = false;
    const uint32_t tile0 = lwg * t.tiles_per_wg;
    for (uint32_t k = 0; k < t.tiles_per_wg; ++k) {
        const uint32_t i = (tile0 + k) * kWG + tid;
        double term[1] = {0.0};
        float w[32];
        // the plain conversion is bound by the reads: packed rows go through the coalescing exchange
        const bool exchanged = !DSS && DT == SOAR_BF16 && t.contiguous;
        if constexpr (!DSS && DT == SOAR_BF16) {
            if (exchanged) load_wave_blocks<DT, 32, true>(t.w, i - (tid & 63u), t.nblk, s_x + (tid >> 6) * (64 * kP), w);
        }
        if (i < t.nblk) {
            float q[32];
            uint32_t nib[4] = {0u, 0u, 0u, 0u};
            if (!exchanged) {
                size_t off;
                if (t.contiguous) {
                    off = (size_t)i * 32;
                } else {
                    const uint32_t row = i / t.bpr;
                    off = (size_t)row * (size_t)t.ld + (size_t)(i - row * t.bpr) * 32;
                }
                // ordinary loads: a lane's four or eight loads share cache lines, which streaming loads would drop
                load_block<DT, false>(t.w, off, w);
                load_block<DT, false>(t.w, off + 16, w + 16);
            }
            uint32_t mbits = 0u;
#pragma unroll
            for (int j = 0; j < 32; ++j) mbits = max(mbits, __float_as_uint(w[j]) & 0x7FFFFFFFu);
            nonfinite = nonfinite || mbits >= 0x7F800000u;
            const float bmax = f_of(mbits);
            // bmax = m 2^ex with m in [0.5, 1): floor(log2 bmax) = ex - 1; the largest E2M1 value is 1.5 * 2^2
            const int ex = __builtin_amdgcn_frexp_expf(bmax);
            const int e0 = mbits == 0u ? 127 : min(max(ex - 1 - 2, -127), 127) + 127;
            int code = e0;
            float err;
            if constexpr (!DSS) {
                const float x0 = e8m0_value(e0);
                mx_assign<false>(w, x0, nib, q);
                err = mx_block_error(w, q, x0);
            } else {
                // the reciprocal shortcut needs the scales X0 beta_k to stay within biased exponents [1, 252]
                const float s_first = e8m0_value(e0) * s_beta[0], s_final = e8m0_value(e0) * s_beta[n_beta - 1];
                const bool mid = ((__float_as_uint(s_first) >> 23) - 2u) < 250u && ((__float_as_uint(s_final) >> 23) - 2u) < 250u;
                const bool fast = __builtin_amdgcn_ballot_w64(!mid) == 0ull;
                if (t.two_pass) {
                    if (fast) mx_search_two_pass<true>(w, e0, s_beta, n_beta, t.radius, s_list, err, code, nib, q);
                    else mx_search_two_pass<false>(w, e0, s_beta, n_beta, t.radius, s_list, err, code, nib, q);
                } else {
                    if (fast) mx_search<true>(w, e0, s_beta, n_beta, t.radius, err, code, nib, q);
                    else mx_search<false>(w, e0, s_beta, n_beta, t.radius, err, code, nib, q);
                }
            }
            term[0] = (double)err;
            u32x4 packed = {nib[0], nib[1], nib[2], nib[3]};
            __builtin_nontemporal_store(packed, reinterpret_cast<u32x4 *>(t.codes) + i);
            __builtin_nontemporal_store((uint8_t)code, t.scales + i);
        }
        tree.add_tile(k, term);
    }
    if (nonfinite) {
        __hip_atomic_fetch_or(&t.ctrl->amax_bits, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0);        // performed before this wave reaches the barrier below
    }
    uint32_t *counters = t.counters;
    if (tid == 0) {
        publish(t.part + lwg, tree.wg[0]);
        s_last = 0u;
    }
    __syncthreads();          // every lane's flag update has been issued before lane 0 counts the workgroup in
    if (tid == 0) s_last = arrive_is_last(counters, &t.ctrl->top[0], t.n_wg, lwg) ? 1u : 0u;
    __syncthreads();
    if (!s_last) return;
    double total;
    trees_of_partials<1>(t.part, t.n_wg, s_tree, &s_stack[0][0], &total);
    if (tid == 0) {
        const uint32_t flag = __hip_atomic_load(&t.ctrl->amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (t.sse) *t.sse = total;
        if (t.status) *t.status = flag ? SOAR_STATUS_NONFINITE : 0;
        t.ctrl->amax_bits = 0u;
    }
    reset_counters(counters, &t.ctrl->top[0]);
}

}  // namespace
