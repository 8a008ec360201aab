// Shared device code of the SOAR kernels (gfx950): launch structures, the E2M1 / E4M3 formats,
// block loads and the coalescing wave exchange, the per-block steps of Eq. 1-2, and the fixed-order
// reductions (wave trees, arrival counters, trees of partials).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>

#include "soar.h"

namespace {


constexpr int kWG = 256;                 // lanes per workgroup = blocks per tile
constexpr int kStage = 4;                // tiles whose block terms are staged in LDS per tree step
constexpr int kMaxPartials = 16384;      // workgroups per tensor, at most
constexpr int kGroupMax = 8;             // tensors per launch
constexpr int64_t kGroupByteCap = (int64_t)1 << 28;   // bytes of weights per launch (beyond the first tensor):
                                                      // a group then fits the 256 MiB last-level cache between passes
constexpr int kSlots = 64;               // first-level arrival counters
constexpr int kSlotStride = 32;          // in uint32: one counter per 128 bytes
constexpr int kKernels = 3;              // absmax, stats, search
constexpr int kLanes = 2;                // streams a batch is spread over
constexpr int kMaxBeta = 4096;           // factors of the quantization-scale grid, at most
constexpr int kMaxIters = 64;
constexpr uint32_t kE4M3Min = 0x01u, kE4M3Max = 0x7Eu;

// Control words of one tensor slot.  soar_quantize* zeroes them once per call;
// after that every kernel leaves its own counters at zero again.
struct Ctrl {
    uint32_t top[4];         // second-level arrival counter of each kernel
    uint32_t amax_bits;      // max |w| as binary32 bits
    float    alpha0;
    float    alpha1;
    uint32_t stopped;        // iterated path: the early stop has fired
    double   N, M;
    double   prev_sse;       // iterated path: error before the iteration now running
    uint64_t epoch;          // one-launch path: advanced by every launch, part of its token (any start value will do)
};
constexpr size_t kCtrlBytes = 256;
static_assert(sizeof(Ctrl) <= kCtrlBytes, "control block");
constexpr size_t kCountersBytes = (size_t)kKernels * kSlots * kSlotStride * 4;
constexpr size_t kSlotMaxBytes = (size_t)kSlots * kSlotStride * 4;
constexpr size_t kZeroedBytes = kCtrlBytes + kCountersBytes + kSlotMaxBytes;   // what k_init clears
constexpr size_t kPartialsBytes = 3 * sizeof(double) * (size_t)kMaxPartials;
constexpr size_t kSlotBytes = kZeroedBytes + kPartialsBytes;                   // per tensor slot
static_assert(kSlotBytes % 256 == 0, "slot size");

// How one pass walks a tensor: workgroups wg_begin .. wg_begin + n_wg - 1 of the grid, tiles_per_wg (a power of
// two) tiles of kWG blocks each.
struct Shape {
    uint32_t tiles_per_wg, n_wg, wg_begin;
};

// One tensor of a launch.
struct Task {
    const void *w;
    uint8_t  *codes, *scales;
    float    *gscale;
    double   *sse;
    int32_t  *status;
    int64_t  ld;             // leading dimension, elements
    uint32_t bpr;            // blocks per row
    uint32_t nblk;           // blocks in the tensor
    uint32_t tiles_per_wg;   // power of two
    uint32_t contiguous;     // ld == cols
    uint32_t wg_begin;       // first workgroup of the grid that works on this tensor
    uint32_t n_wg;           // how many do
    // workspace of the slot
    Ctrl     *ctrl;
    uint32_t *counters;      // [kKernels][kSlots] arrival counters, kSlotStride apart
    uint32_t *slot_max;      // [kSlots] partial maxima of the absmax kernel, kSlotStride apart
    double   *part;          // [3][kMaxPartials] partial sums N, M, error
    float    *rho;           // [nblk] a / b of the current state, or -Delta^d where b == 0
    const float *amax_in;    // supplied maximum (plain NVFP4 only), or null: measured by k_absmax
    Shape    absmax, search; // shapes of k_absmax and k_search (tiles_per_wg, wg_begin, n_wg above: every other kernel)
    int32_t  *iters_run;     // iterated path, may be null
    double   *trace;         // iterated path, may be null: iters+1 errors
};

struct Batch {
    Task     t[kGroupMax];
    uint32_t n;
    int32_t  radius;
    int32_t  full_search;
    unsigned long long *search_stats;   // null, or four counters (see count_search): diagnostics only
    // iterated path
    int32_t  iter_t;         // iteration this launch carries out
    int32_t  n_beta;
    int32_t  dd_mode;
    float    beta_lo, beta_hi;
    float    early_stop_rel;
    int32_t  arm;            // soar_method of the iterated path: SOAR, CJSO_ONLY or DSS_ONLY
};

typedef Task Geom;           // the addressing fields are all block_offset needs

// ------------------------------------------------------------------ formats
__device__ __forceinline__ float f_of(uint32_t u) { return __uint_as_float(u); }

// positive E4M3 code -> value.  code<<20 read as binary32 has the same exponent
// and mantissa fields with a bias off by 120, subnormals included.
__device__ __forceinline__ float e4m3_value(uint32_t code) { return f_of(code << 20) * 0x1p120f; }

// Appendix D: round to nearest even onto E4M3, clip to [2^-9, 448]
__device__ __forceinline__ uint32_t e4m3_project(float y)
{
    y = fminf(fmaxf(y, 0.0f), 448.0f);            // NaN -> 0
    uint32_t u = __float_as_uint(y);
    u += 0x7FFFFu + ((u >> 20) & 1u);             // RNE to 3 mantissa bits
    uint32_t normal = (u >> 20) - (120u << 3);
    uint32_t sub = (uint32_t)__float2int_rn(y * 512.0f);
    uint32_t code = (y >= 0x1p-6f) ? normal : sub;
    return min(max(code, kE4M3Min), kE4M3Max);
}

// Eq. 2 on eight values: hardware E2M1 conversion (round to nearest even,
// saturating, sign kept on zero), element 0 in the lowest nibble.
__device__ __forceinline__ uint32_t fp4x8(const float *x)
{
    uint32_t r = 0;
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, x[0], x[1], 1.0f, 0);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, x[2], x[3], 1.0f, 1);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, x[4], x[5], 1.0f, 2);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, x[6], x[7], 1.0f, 3);
    return r;
}

__device__ __forceinline__ void fp4x8_values(uint32_t r, float *q)
{
    auto v0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r, 1.0f, 0);
    auto v1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r, 1.0f, 1);
    auto v2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r, 1.0f, 2);
    auto v3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r, 1.0f, 3);
    q[0] = v0[0]; q[1] = v0[1]; q[2] = v1[0]; q[3] = v1[1];
    q[4] = v2[0]; q[5] = v2[1]; q[6] = v3[0]; q[7] = v3[1];
}

// ------------------------------------------------------------------ loads
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// The first two passes read the weights with ordinary loads, so that a launch group (at most
// 256 MiB) stays in the last-level cache for the pass that follows; the search pass, the last
// reader, streams them.
constexpr bool kStreamAbsmax = false, kStreamStats = false, kStreamSearch = true;

// 16 bytes; STREAM = nontemporal (no reuse expected by this kernel)
template <bool STREAM>
__device__ __forceinline__ u32x4 load16(const void *p)
{
    if constexpr (STREAM) return __builtin_nontemporal_load(static_cast<const u32x4 *>(p));
    else return *static_cast<const u32x4 *>(p);
}

template <int DT, bool STREAM = false>
__device__ __forceinline__ void load_block(const void *base, size_t elem_off, float w[16])
{
    if constexpr (DT == SOAR_BF16) {
        const uint16_t *p = static_cast<const uint16_t *>(base) + elem_off;
        const u32x4 v0 = load16<STREAM>(p), v1 = load16<STREAM>(p + 8);
        uint32_t u[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            w[2 * k] = f_of(u[k] << 16);
            w[2 * k + 1] = f_of(u[k] & 0xFFFF0000u);
        }
    } else {
        const float *p = static_cast<const float *>(base) + elem_off;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u32x4 v = load16<STREAM>(p + 4 * k);
            w[4 * k] = f_of(v.x); w[4 * k + 1] = f_of(v.y); w[4 * k + 2] = f_of(v.z); w[4 * k + 3] = f_of(v.w);
        }
    }
}

// The 64 consecutive blocks of a wave lie in one contiguous range when the rows of the tensor are
// packed (ld == cols): 64 * P pieces of 16 bytes.  A lane that reads or writes its own 32, 64 or 128
// contiguous bytes touches every cache line of the range with every instruction; the wave moves the
// range in fully coalesced pieces instead (lane l takes pieces l, l + 64, ...) and each lane finds
// the P pieces of its own block in a wave-private LDS region of 64 * P pieces.  Inside a block's
// slots the pieces are rotated by the block's row of 256 bytes, so that neither side of the exchange
// has bank conflicts.  A wave's LDS operations execute in order: no workgroup barrier is needed.
// Data movement only.  `have` = pieces of the range that exist (the tensor may end inside it).
template <int P>
__device__ __forceinline__ uint32_t exchange_slot(uint32_t block, uint32_t piece)
{
    static_assert(P == 2 || P == 4 || P == 8, "block of 32, 64 or 128 bytes");
    return block * (uint32_t)P + ((piece + block / (uint32_t)(16 / P)) & (uint32_t)(P - 1));
}

template <int P, bool STREAM>
__device__ __forceinline__ void load_wave_pieces(const u32x4 *range, uint32_t have, u32x4 *s_wave, u32x4 v[P])
{
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const uint32_t idx = (uint32_t)p * 64u + lane;
        v[p] = u32x4{0u, 0u, 0u, 0u};
        if (idx < have) v[p] = load16<STREAM>(range + idx);
    }
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const uint32_t idx = (uint32_t)p * 64u + lane;
        s_wave[exchange_slot<P>(idx / (uint32_t)P, idx % (uint32_t)P)] = v[p];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int p = 0; p < P; ++p) v[p] = s_wave[exchange_slot<P>(lane, (uint32_t)p)];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();                     // the next exchange writes these slots again
}

template <int P, bool STREAM>
__device__ __forceinline__ void store_wave_pieces(u32x4 *range, uint32_t have, u32x4 *s_wave, const u32x4 v[P])
{
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int p = 0; p < P; ++p) s_wave[exchange_slot<P>(lane, (uint32_t)p)] = v[p];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const uint32_t idx = (uint32_t)p * 64u + lane;
        const u32x4 x = s_wave[exchange_slot<P>(idx / (uint32_t)P, idx % (uint32_t)P)];
        if (idx < have) {
            if constexpr (STREAM) __builtin_nontemporal_store(x, range + idx);
            else range[idx] = x;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// 16-byte pieces of one block of NELEM elements
template <int DT, int NELEM>
constexpr int pieces_per_block() { return NELEM * (DT == SOAR_BF16 ? 2 : 4) / 16; }

// pieces of the wave's range [wave_first, wave_first + 64) that lie inside a tensor of nblk blocks
template <int P>
__device__ __forceinline__ uint32_t wave_pieces(uint32_t wave_first, uint32_t nblk)
{
    return wave_first < nblk ? min(64u, nblk - wave_first) * (uint32_t)P : 0u;
}

// load_block for every lane of a wave at once through the coalescing exchange: w[] ends up exactly
// as load_block leaves it; blocks at or beyond nblk read as zeros
template <int DT, int NELEM, bool STREAM>
__device__ __forceinline__ void load_wave_blocks(const void *base, uint32_t wave_first, uint32_t nblk,
                                                 u32x4 *s_wave, float w[NELEM])
{
    constexpr int P = pieces_per_block<DT, NELEM>();
    u32x4 v[P];
    load_wave_pieces<P, STREAM>(static_cast<const u32x4 *>(base) + (size_t)wave_first * P, wave_pieces<P>(wave_first, nblk),
                                s_wave, v);
    if constexpr (DT == SOAR_BF16) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const uint32_t u[4] = {v[p].x, v[p].y, v[p].z, v[p].w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                w[8 * p + 2 * k] = f_of(u[k] << 16);
                w[8 * p + 2 * k + 1] = f_of(u[k] & 0xFFFF0000u);
            }
        }
    } else {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            w[4 * p] = f_of(v[p].x); w[4 * p + 1] = f_of(v[p].y); w[4 * p + 2] = f_of(v[p].z); w[4 * p + 3] = f_of(v[p].w);
        }
    }
}

// NELEM values of a lane's block to the output element type and out through the exchange
template <int DT, int NELEM>
__device__ __forceinline__ void store_wave_blocks(void *base, uint32_t wave_first, uint32_t nblk, u32x4 *s_wave,
                                                  const float v[NELEM])
{
    constexpr int P = pieces_per_block<DT, NELEM>();
    u32x4 x[P];
    if constexpr (DT == SOAR_BF16) {
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        typedef float f2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int p = 0; p < P; ++p) {
            uint32_t u[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                f2 in = {v[8 * p + 2 * k], v[8 * p + 2 * k + 1]};
                bf2 o = __builtin_convertvector(in, bf2);     // round to nearest even
                __builtin_memcpy(&u[k], &o, 4);
            }
            x[p] = u32x4{u[0], u[1], u[2], u[3]};
        }
    } else {
#pragma unroll
        for (int p = 0; p < P; ++p)
            x[p] = u32x4{__float_as_uint(v[4 * p]), __float_as_uint(v[4 * p + 1]), __float_as_uint(v[4 * p + 2]),
                         __float_as_uint(v[4 * p + 3])};
    }
    // streaming stores: in the probe ordinary ones are level or slightly ahead at 64 bytes per lane, in the
    // dequantization kernels they are 8 % behind (the written lines linger in the caches)
    store_wave_pieces<P, true>(static_cast<u32x4 *>(base) + (size_t)wave_first * P, wave_pieces<P>(wave_first, nblk), s_wave, x);
}

__device__ __forceinline__ size_t block_offset(const Geom &g, uint32_t i)
{
    if (g.contiguous) return (size_t)i * 16;
    uint32_t row = i / g.bpr;
    uint32_t cb = i - row * g.bpr;
    return (size_t)row * (size_t)g.ld + (size_t)cb * 16;
}

// same, with the addressing fields already in registers
__device__ __forceinline__ size_t block_offset(bool contiguous, uint32_t bpr, int64_t ld, uint32_t i)
{
    if (contiguous) return (size_t)i * 16;
    uint32_t row = i / bpr;
    uint32_t cb = i - row * bpr;
    return (size_t)row * (size_t)ld + (size_t)cb * 16;
}

// ------------------------------------------------------------------ per-block steps
// Q = Q_FP4(W / scale) as a product with the correctly rounded reciprocal
__device__ __forceinline__ void assign_codes(const float w[16], float scale, uint32_t nib[2], float q[16])
{
    float r = 1.0f / scale;
    float x[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) x[j] = w[j] * r;
    nib[0] = fp4x8(x);
    nib[1] = fp4x8(x + 8);
    fp4x8_values(nib[0], q);
    fp4x8_values(nib[1], q + 8);
}

// Eq. 8 for one candidate scale s = alpha * d: ascending chain of fused operations.
// w - q*s is formed as fma(q, -s, w): the product's sign flips exactly, and negating the
// one scale instead of the sixteen codes leaves nothing for the compiler to materialise.
__device__ __forceinline__ float block_error(const float w[16], const float q[16], float s)
{
    const float ns = -s;
    float err = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        float e = __builtin_fmaf(q[j], ns, w[j]);
        err = __builtin_fmaf(e, e, err);
    }
    return err;
}

__device__ __forceinline__ void block_sums(const float w[16], const float q[16], float &a, float &b)
{
    a = 0.0f; b = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        a = __builtin_fmaf(w[j], q[j], a);
        b = __builtin_fmaf(q[j], q[j], b);
    }
}

// Eq. 1 block scale and Eq. 2 assignment under (alpha0, Delta0)
__device__ __forceinline__ void block_init(const float w[16], float alpha0, float alpha0_m,
                                           uint32_t &c0, float &delta0, uint32_t nib[2], float q[16])
{
    float bmax = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) bmax = fmaxf(bmax, fabsf(w[j]));
    c0 = e4m3_project(bmax / alpha0_m);
    delta0 = e4m3_value(c0);
    assign_codes(w, alpha0 * delta0, nib, q);
}

// ------------------------------------------------------------------ reductions
// Adjacent-pair tree over the 64 lanes of a wave; the result is uniform.
// Inside a row of 16 lanes the partner values come through DPP (lane^1, lane^2,
// then the mirrored half-row and row, whose lanes already hold equal sums);
// the four row sums are combined as (r0+r1)+(r2+r3).
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double readlane_f64(double v, int lane)
{
    int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_pair_tree(double v)
{
    v = v + dpp_f64<0xB1>(v);      // quad_perm [1,0,3,2]
    v = v + dpp_f64<0x4E>(v);      // quad_perm [2,3,0,1]
    v = v + dpp_f64<0x141>(v);     // row_half_mirror
    v = v + dpp_f64<0x140>(v);     // row_mirror
    const double r0 = readlane_f64(v, 0), r1 = readlane_f64(v, 16);
    const double r2 = readlane_f64(v, 32), r3 = readlane_f64(v, 48);
    return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t m)
{
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) m = max(m, (uint32_t)__shfl_xor((int)m, s, 64));
    return m;
}

// Inter-workgroup hand-off without cache-wide fences.  A workgroup publishes its
// partial result with agent-scope atomics (performed at the point of coherence),
// waits until they have completed, and then counts itself in with relaxed
// agent-scope atomics; the workgroup that completes the count reads the partials
// back with agent-scope atomic loads.  Arrival is counted on two levels (kSlots
// first-level counters, one top counter) because read-modify-writes on a single
// address serialise at roughly ten nanoseconds each.
//
// What the hand-off rests on (stronger than the HIP memory model's relaxed atomics promise by
// themselves; true of gfx950 and of the code the compiler emits for these builtins):
//  (1) an agent-scope atomic store or read-modify-write is performed at the memory side, beyond the
//      per-XCD L2, and the wave's vmcnt counts it until it has been performed there; s_waitcnt(0)
//      therefore returns only when everything the lane published is visible to every workgroup;
//  (2) the compiler keeps the order publish -> s_waitcnt -> count: the workgroup-scope release fence
//      in between forbids moving the stores below it;
//  (3) ONE lane publishes and counts (the publishing lane's own vmcnt is the one that is waited on);
//      a workgroup whose publishing is spread over lanes must bring them together (a workgroup barrier,
//      whose stores have then completed per lane) before the counting lane counts;
//  (4) the reader's agent-scope atomic loads are issued after its own fetch_add has returned (its
//      result decides the branch they sit in) and bypass the non-coherent caches.
// The counting itself is plain arithmetic, stated separately so that it can be checked on the host:
struct ArrivalPlan {
    uint32_t ns;         // first-level counters in use
    uint32_t slot;       // the one this workgroup counts on
    uint32_t expected;   // how many workgroups count on that one
};
__host__ __device__ inline ArrivalPlan arrival_plan(uint32_t G, uint32_t lwg)
{
    ArrivalPlan p;
    p.ns = G < (uint32_t)kSlots ? G : (uint32_t)kSlots;
    p.slot = lwg % p.ns;
    p.expected = (G - p.slot + p.ns - 1) / p.ns;      // workgroups lwg' < G with lwg' % ns == slot
    return p;
}

__device__ __forceinline__ void publish(double *p, double v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// called by one lane of the workgroup -- the lane that published; true for exactly one of the tensor's
// G workgroups: the one whose increment completes its first-level counter and then the top counter
__device__ __forceinline__ bool arrive_is_last(uint32_t *slots, uint32_t *top, uint32_t G, uint32_t lwg)
{
    const ArrivalPlan plan = arrival_plan(G, lwg);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);          // what this lane published has completed
    uint32_t t = __hip_atomic_fetch_add(slots + plan.slot * kSlotStride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t != plan.expected - 1) return false;
    uint32_t t2 = __hip_atomic_fetch_add(top, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return t2 == plan.ns - 1;
}

// the last workgroup puts the counters back to zero for the next launch
__device__ __forceinline__ void reset_counters(uint32_t *slots, uint32_t *top)
{
    if (threadIdx.x < kSlots) slots[threadIdx.x * kSlotStride] = 0u;
    if (threadIdx.x == 0) *top = 0u;
}

// Adjacent-pair trees over NV arrays of per-workgroup partial sums (array n starts at part + n * kMaxPartials,
// entries 0..P), zero-padded to a power of two.  All kWG lanes of the workgroup must call; result[] is valid in
// lane 0.  Chunks of 8*kWG (4*kWG for three arrays) partials: that many adjacent ones per lane in registers, the DPP tree over a wave's lanes,
// the four wave sums through LDS (lds: 4 NV doubles), and a binary-counter stack over the chunks (stack: 32
// doubles per array).  The loads of all arrays are issued together: the last workgroup pays one trip to
// memory and two barriers per chunk, whatever NV.
template <int NV>
__device__ void trees_of_partials(const double *part, uint32_t P, double *lds, double *stack, double result[NV])
{
    constexpr uint32_t kPerLane = NV >= 3 ? 4 : 8;       // adjacent partials per lane and array: 24 to 32 registers
    static_assert(kWG == 256, "four wave sums per chunk");
    uint32_t P2 = 1;
    while (P2 < P) P2 <<= 1;
    const uint32_t C = P2 > (uint32_t)kWG ? (P2 / kWG < kPerLane ? P2 / kWG : kPerLane) : 1;
    const uint32_t chunk = C * kWG;
    const uint32_t nchunks = P2 > chunk ? P2 / chunk : 1;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
#pragma unroll
    for (int n = 0; n < NV; ++n) result[n] = 0.0;
    for (uint32_t ch = 0; ch < nchunks; ++ch) {
        double v[NV][kPerLane];
#pragma unroll
        for (int n = 0; n < NV; ++n)
#pragma unroll
            for (uint32_t k = 0; k < kPerLane; ++k) {
                const uint32_t idx = ch * chunk + tid * C + k;
                v[n][k] = (k < C && idx < P)
                              ? __hip_atomic_load(part + (size_t)n * kMaxPartials + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                              : 0.0;
            }
        double w[NV];
#pragma unroll
        for (int n = 0; n < NV; ++n) {
#pragma unroll
            for (uint32_t s = 1; s < kPerLane; s <<= 1)
#pragma unroll
                for (uint32_t k = 0; k < kPerLane; k += 2 * s) v[n][k] = v[n][k] + v[n][k + s];
            w[n] = wave_pair_tree(v[n][0]);
        }
        __syncthreads();          // lds may alias what the caller used before; lane 0 has read the chunk before
        if (lane == 0) {
#pragma unroll
            for (int n = 0; n < NV; ++n) lds[n * 4 + wave] = w[n];
        }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int n = 0; n < NV; ++n) {
                double x = (lds[n * 4] + lds[n * 4 + 1]) + (lds[n * 4 + 2] + lds[n * 4 + 3]);
                uint32_t lvl = 0;
                while ((ch >> lvl) & 1u) { x = stack[n * 32 + lvl] + x; ++lvl; }
                stack[n * 32 + lvl] = x;
                result[n] = x;
            }
        }
    }
}

// which tensor of the launch this workgroup works on, and its index there
__device__ __forceinline__ uint32_t find_task(const Batch &b, uint32_t &lwg)
{
    const uint32_t id = blockIdx.x;
    uint32_t k = 0;
    for (uint32_t j = 1; j < b.n; ++j)
        if (id >= b.t[j].wg_begin) k = j;
    lwg = id - b.t[k].wg_begin;
    return k;
}

// the same for a pass with a shape of its own
__device__ __forceinline__ uint32_t find_task(const Batch &b, Shape Task::*which, uint32_t &lwg)
{
    const uint32_t id = blockIdx.x;
    uint32_t k = 0;
    for (uint32_t j = 1; j < b.n; ++j)
        if (id >= (b.t[j].*which).wg_begin) k = j;
    lwg = id - (b.t[k].*which).wg_begin;
    return k;
}

}  // namespace
