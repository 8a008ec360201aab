// SOAR NVFP4 weight quantization for MI355X (gfx950): HIP kernels and C-ABI.
//
// Path (arXiv 2605.12245, Algorithm 1 with T = 1 and beta = 1), three streaming
// kernels per group of tensors:
//   absmax   max|W|                                     -> alpha0       (Eq. 1)
//   stats    per block: Delta0, Q0, a = sum w q, b = sum q^2            (Eq. 1-2)
//            tensor:    N = sum a Delta0, M = sum b Delta0^2 -> alpha1  (Eq. 5)
//   search   per block: Delta* = a/(alpha1 b) (Eq. 6), centre = E4M3(Delta*)
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
#include <cstring>
#include <vector>

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
};
constexpr size_t kCtrlBytes = 256;
static_assert(sizeof(Ctrl) <= kCtrlBytes, "control block");
constexpr size_t kCountersBytes = (size_t)kKernels * kSlots * kSlotStride * 4;
constexpr size_t kSlotMaxBytes = (size_t)kSlots * kSlotStride * 4;
constexpr size_t kZeroedBytes = kCtrlBytes + kCountersBytes + kSlotMaxBytes;   // what k_init clears
constexpr size_t kPartialsBytes = 3 * sizeof(double) * (size_t)kMaxPartials;
constexpr size_t kSlotBytes = kZeroedBytes + kPartialsBytes;                   // per tensor slot
static_assert(kSlotBytes % 256 == 0, "slot size");

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
    int32_t  *iters_run;     // iterated path, may be null
    double   *trace;         // iterated path, may be null: iters+1 errors
};

struct Batch {
    Task     t[kGroupMax];
    uint32_t n;
    int32_t  radius;
    int32_t  full_search;
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
__device__ __forceinline__ void publish(double *p, double v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// called by one lane of the workgroup; true for exactly one of the tensor's G workgroups
__device__ __forceinline__ bool arrive_is_last(uint32_t *slots, uint32_t *top, uint32_t G, uint32_t lwg)
{
    const uint32_t ns = G < (uint32_t)kSlots ? G : (uint32_t)kSlots;
    const uint32_t slot = lwg % ns;
    const uint32_t expected = (G - slot + ns - 1) / ns;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);          // what this lane published has completed
    uint32_t t = __hip_atomic_fetch_add(slots + slot * kSlotStride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t != expected - 1) return false;
    uint32_t t2 = __hip_atomic_fetch_add(top, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return t2 == ns - 1;
}

// the last workgroup puts the counters back to zero for the next launch
__device__ __forceinline__ void reset_counters(uint32_t *slots, uint32_t *top)
{
    if (threadIdx.x < kSlots) slots[threadIdx.x * kSlotStride] = 0u;
    if (threadIdx.x == 0) *top = 0u;
}

// Adjacent-pair tree over the per-workgroup partial sums part[0..P), zero-padded
// to a power of two.  All lanes of the workgroup must call; the result is valid
// in lane 0.  Chunks of 8*kWG partials are folded (8 per lane in registers, then
// LDS) and combined with a binary-counter stack.
__device__ double tree_of_partials(const double *part, uint32_t P, double *lds /* kWG */, double *stack /* 16 */)
{
    constexpr uint32_t kPerLane = 8;
    uint32_t P2 = 1;
    while (P2 < P) P2 <<= 1;
    const uint32_t C = P2 > (uint32_t)kWG ? (P2 / kWG < kPerLane ? P2 / kWG : kPerLane) : 1;
    const uint32_t chunk = C * kWG;
    const uint32_t nchunks = P2 > chunk ? P2 / chunk : 1;
    const uint32_t tid = threadIdx.x;
    double result = 0.0;
    for (uint32_t ch = 0; ch < nchunks; ++ch) {
        double v[kPerLane];
#pragma unroll
        for (uint32_t k = 0; k < kPerLane; ++k) {
            const uint32_t idx = ch * chunk + tid * C + k;
            v[k] = (k < C && idx < P)
                       ? __hip_atomic_load(part + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                       : 0.0;
        }
#pragma unroll
        for (uint32_t s = 1; s < kPerLane; s <<= 1)
#pragma unroll
            for (uint32_t k = 0; k < kPerLane; k += 2 * s) v[k] = v[k] + v[k + s];
        __syncthreads();
        lds[tid] = v[0];
        __syncthreads();
        for (uint32_t n = kWG; n > 1; n >>= 1) {
            double t = 0.0;
            if (tid < n / 2) t = lds[2 * tid] + lds[2 * tid + 1];
            __syncthreads();
            if (tid < n / 2) lds[tid] = t;
            __syncthreads();
        }
        if (tid == 0) {
            double x = lds[0];
            uint32_t lvl = 0;
            while ((ch >> lvl) & 1u) { x = stack[lvl] + x; ++lvl; }
            stack[lvl] = x;
            result = x;
        }
    }
    return result;
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

// ------------------------------------------------------------------ kernels
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

// ------------------------------------------------------------------ iterated path
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

// largest E4M3 code in [0x01, 0x7E] whose value does not exceed y (0x01 if none does)
__device__ __forceinline__ int e4m3_floor_code(float y)
{
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
    __shared__ double s_wave[3][4];
    __shared__ double s_stack[3][32];
    __shared__ double s_tree[kWG];
    __shared__ uint32_t s_last;

    uint32_t lwg;
    const Task t = batch.t[find_task(batch, lwg)];
    const uint32_t tid = threadIdx.x;
    const uint32_t amax_bits = t.ctrl->amax_bits;
    const bool degenerate = amax_bits == 0u || amax_bits >= 0x7F800000u;
    const float alpha0 = f_of(amax_bits) / 2688.0f;
    const float alpha0_m = alpha0 * 6.0f;

    TileTree<3> tree{s_wave, s_stack};
    const uint32_t tile0 = lwg * t.tiles_per_wg;
    for (uint32_t k = 0; k < t.tiles_per_wg; ++k) {
        const uint32_t i = (tile0 + k) * kWG + tid;
        double term[3] = {0.0, 0.0, 0.0};
        if (i < t.nblk) {
            float rho = 0.0f;
            if (!degenerate) {
                float w[16], q[16];
                uint32_t nib[2], c0;
                float delta0, a, b;
                load_block<DT>(t.w, block_offset(t, i), w);
                block_init(w, alpha0, alpha0_m, c0, delta0, nib, q);
                block_sums(w, q, a, b);
                term[0] = (double)a * (double)delta0;
                term[1] = ((double)b * (double)delta0) * (double)delta0;
                term[2] = (double)block_error(w, q, alpha0 * delta0);
                rho = (b == 0.0f || batch.arm == SOAR_METHOD_DSS_ONLY) ? -delta0 : a / b;
            }
            t.rho[i] = rho;
        }
        tree.add_tile(k, term);
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
    const double N = tree_of_partials(t.part, t.n_wg, s_tree, s_stack[0]);
    const double M = tree_of_partials(t.part + kMaxPartials, t.n_wg, s_tree, s_stack[1]);
    const double E = tree_of_partials(t.part + 2 * kMaxPartials, t.n_wg, s_tree, s_stack[2]);
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
    const bool one_scale = batch.arm == SOAR_METHOD_CJSO_ONLY;
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
                if (one_scale) {
                    // Sec. 3.2 alone: the projected scale assigns the codes and is stored; nothing to search
                    best_code = c0;
                    const float sd = alpha * e4m3_value((uint32_t)c0);
                    assign_codes(w, sd, best_nib, q);
                    best_err = block_error(w, q, sd);
                } else if (two_pass) {
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
    const double N = tree_of_partials(t.part, t.n_wg, s_tree, s_stack[0]);
    const double M = tree_of_partials(t.part + kMaxPartials, t.n_wg, s_tree, s_stack[1]);
    const double cur = tree_of_partials(t.part + 2 * kMaxPartials, t.n_wg, s_tree, s_stack[2]);
    if (tid == 0) {
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
    reset_counters(counters, &t.ctrl->top[2]);
}

// ------------------------------------------------------------------ MXFP4
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
        float m = mx_block_error(w, q, x0);
        for (int c = 1; c <= 2 * radius; ++c) m = fminf(m, mx_block_error(w, q, e8m0_value(mx_candidate(e0, c))));
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
            float m = mx_block_error(w, q, x0);
            for (int c = 1; c <= 2 * radius; ++c) m = fminf(m, mx_block_error(w, q, e8m0_value(mx_candidate(e0, c))));
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
    __shared__ u32x4 s_x[DSS ? 1 : kWG * kP];          // load_wave_blocks: one region per wave
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
        const bool exchanged = !DSS && t.contiguous;
        if constexpr (!DSS) {
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
    const double total = tree_of_partials(t.part, t.n_wg, s_tree, s_stack[0]);
    if (tid == 0) {
        const uint32_t flag = __hip_atomic_load(&t.ctrl->amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (t.sse) *t.sse = total;
        if (t.status) *t.status = flag ? SOAR_STATUS_NONFINITE : 0;
        t.ctrl->amax_bits = 0u;
    }
    reset_counters(counters, &t.ctrl->top[0]);
}

template <int DT>
__global__ __launch_bounds__(kWG) void k_mx_dequant(const uint8_t *codes, const uint8_t *scales, uint32_t nblk,
                                                    uint32_t bpr, int64_t ld, uint32_t contiguous, void *out)
{
    constexpr int kP = pieces_per_block<DT, 32>();
    __shared__ u32x4 s_x[kWG * kP];                    // store_wave_blocks: one region per wave
    const uint32_t i = blockIdx.x * kWG + threadIdx.x;
    const uint32_t wave_first = i - (threadIdx.x & 63u);
    if (wave_first >= nblk) return;
    const bool inside = i < nblk;
    const uint32_t e = inside ? (uint32_t)__builtin_nontemporal_load(scales + i) : 127u;
    const bool skip = e == 255u;                        // not a scale: the block's output is left alone
    float v[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) v[j] = 0.0f;
    if (inside && !skip) {
        const float s = e8m0_value((int)e);
        const u32x4 nb = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(codes) + i);
        fp4x8_values(nb.x, v);
        fp4x8_values(nb.y, v + 8);
        fp4x8_values(nb.z, v + 16);
        fp4x8_values(nb.w, v + 24);
#pragma unroll
        for (int j = 0; j < 32; ++j) v[j] = v[j] * s;
    }
    // packed rows: the wave writes its 64 blocks in coalesced pieces, unless one of them is to be skipped
    if (contiguous && __builtin_amdgcn_ballot_w64(skip) == 0ull) {
        store_wave_blocks<DT, 32>(out, wave_first, nblk, s_x + (threadIdx.x >> 6) * (64 * kP), v);
        return;
    }
    if (!inside || skip) return;
    size_t off;
    if (contiguous) {
        off = (size_t)i * 32;
    } else {
        const uint32_t row = i / bpr;
        off = (size_t)row * (size_t)ld + (size_t)(i - row * bpr) * 32;
    }
    if constexpr (DT == SOAR_BF16) {
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        typedef float f2 __attribute__((ext_vector_type(2)));
        uint32_t u[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            f2 in = {v[2 * k], v[2 * k + 1]};
            bf2 o = __builtin_convertvector(in, bf2);     // round to nearest even
            __builtin_memcpy(&u[k], &o, 4);
        }
        uint4 *p = reinterpret_cast<uint4 *>(static_cast<uint16_t *>(out) + off);
#pragma unroll
        for (int k = 0; k < 4; ++k) p[k] = make_uint4(u[4 * k], u[4 * k + 1], u[4 * k + 2], u[4 * k + 3]);
    } else {
        float4 *p = reinterpret_cast<float4 *>(static_cast<float *>(out) + off);
#pragma unroll
        for (int k = 0; k < 8; ++k) p[k] = make_float4(v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]);
    }
}

// Eq. 3
template <int DT>
__global__ __launch_bounds__(kWG) void k_dequant(const uint8_t *codes, const uint8_t *scales,
                                                 const float *d_global_scale, Task g, void *out)
{
    constexpr int kP = pieces_per_block<DT, 16>();
    __shared__ u32x4 s_x[kWG * kP];                    // store_wave_blocks: one region per wave
    const uint32_t i = blockIdx.x * kWG + threadIdx.x;
    const uint32_t wave_first = i - (threadIdx.x & 63u);
    if (wave_first >= g.nblk) return;
    float v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = 0.0f;
    if (i < g.nblk) {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        const float s = *d_global_scale * e4m3_value(__builtin_nontemporal_load(scales + i));
        const u32x2 nb = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(codes) + i);
        float q[16];
        fp4x8_values(nb.x, q);
        fp4x8_values(nb.y, q + 8);
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = q[j] * s;
    }
    if (g.contiguous) {
        // packed rows: the wave writes its 64 blocks in coalesced pieces (all of its lanes take part)
        store_wave_blocks<DT, 16>(out, wave_first, g.nblk, s_x + (threadIdx.x >> 6) * (64 * kP), v);
        return;
    }
    if (i >= g.nblk) return;
    const size_t off = block_offset(g, i);
    if constexpr (DT == SOAR_BF16) {
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        typedef float f2 __attribute__((ext_vector_type(2)));
        uint32_t u[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            f2 in = {v[2 * k], v[2 * k + 1]};
            bf2 o = __builtin_convertvector(in, bf2);     // round to nearest even
            __builtin_memcpy(&u[k], &o, 4);
        }
        uint4 *p = reinterpret_cast<uint4 *>(static_cast<uint16_t *>(out) + off);
        p[0] = make_uint4(u[0], u[1], u[2], u[3]);
        p[1] = make_uint4(u[4], u[5], u[6], u[7]);
    } else {
        float4 *p = reinterpret_cast<float4 *>(static_cast<float *>(out) + off);
#pragma unroll
        for (int k = 0; k < 4; ++k) p[k] = make_float4(v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]);
    }
}

__global__ void k_zero_f64(double *p) { *p = 0.0; }

// Eq. 4 for stored codes and scales.  Every workgroup ends with one binary64 atomic addition to the
// result; additions to one address are served one after the other (thousands of them cost more than
// the reads of a whole tensor), so the workgroups are few and large: 16 waves each, at most kReconGrid.
constexpr int kReconWG = 1024;
constexpr uint32_t kReconGrid = 512;
template <int DT>
__global__ __launch_bounds__(kReconWG) void k_recon(Task g, const uint8_t *codes, const uint8_t *scales,
                                                    const float *d_global_scale, double *d_sse)
{
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    constexpr int kP = pieces_per_block<DT, 16>();
    __shared__ u32x4 s_x[kReconWG * kP];               // load_wave_blocks: one region per wave
    __shared__ double s_wave[kReconWG / 64];
    const uint32_t tid = threadIdx.x;
    const float alpha = *d_global_scale;
    double sse = 0.0;
    // the workgroups in flight sweep one contiguous window of memory
    for (uint32_t first = blockIdx.x * kReconWG; first < g.nblk; first += gridDim.x * kReconWG) {
        const uint32_t i = first + tid;
        const bool inside = i < g.nblk;
        float w[16], q[16];
        if (g.contiguous) load_wave_blocks<DT, 16, true>(g.w, i - (tid & 63u), g.nblk, s_x + (tid >> 6) * (64 * kP), w);
        else if (inside) load_block<DT, false>(g.w, block_offset(g, i), w);
        if (inside) {
            const u32x2 nb = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(codes) + i);
            fp4x8_values(nb.x, q);
            fp4x8_values(nb.y, q + 8);
            sse += (double)block_error(w, q, alpha * e4m3_value(__builtin_nontemporal_load(scales + i)));
        }
    }
    sse = wave_pair_tree(sse);
    if ((tid & 63) == 0) s_wave[tid >> 6] = sse;
    __syncthreads();
    if (tid < 64) {
        double v = tid < kReconWG / 64 ? s_wave[tid] : 0.0;
        v = wave_pair_tree(v);
        if (tid == 0) atomicAdd(d_sse, v);
    }
}

__global__ void k_e2m1_round(const float *x, int64_t n, uint8_t *out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (uint8_t)(__builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, x[i], 0.0f, 1.0f, 0) & 0xFu);
}

__global__ void k_e4m3_project(const float *x, int64_t n, uint8_t *out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (uint8_t)e4m3_project(x[i]);
}

__global__ void k_rcp_midrange(const float *x, int64_t n, float *out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = rcp_midrange(x[i]);
}

// ------------------------------------------------------------------ host side
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
        if (!g_timing.enabled) return;
        if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) { e0 = e1 = nullptr; return; }
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
    if (p->streams < 0 || p->streams > kLanes) return false;
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

// addressing and launch shape of one tensor; the workspace fields stay unset
Task make_task(const void *w, int64_t rows, int64_t cols, int64_t ld, uint32_t forced_tpw)
{
    Task t;
    std::memset(&t, 0, sizeof(t));
    t.w = w;
    t.ld = ld;
    t.bpr = (uint32_t)(cols / 16);
    t.nblk = (uint32_t)(rows * (cols / 16));
    t.contiguous = (ld == cols) ? 1u : 0u;
    const uint32_t tiles = (t.nblk + kWG - 1) / kWG;
    uint32_t tpw = 1;
    while (tpw < (uint32_t)kStage && tpw * 2 <= tiles) tpw <<= 1;
    if (forced_tpw) tpw = forced_tpw;
    while ((tiles + tpw - 1) / tpw > (uint32_t)kMaxPartials) tpw <<= 1;
    t.tiles_per_wg = tpw;
    t.n_wg = (tiles + tpw - 1) / tpw;
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

int32_t group_end(int32_t n, const soar_tensor_desc *descs, int32_t first)
{
    int64_t bytes = weight_bytes(descs[first]);
    int32_t j = first + 1;
    while (j < n && j - first < kGroupMax && descs[j].dtype == descs[first].dtype &&
           bytes + weight_bytes(descs[j]) <= kGroupByteCap) {
        bytes += weight_bytes(descs[j]);
        ++j;
    }
    return j;
}

// most per-block workspace any one launch of the batch needs
size_t max_group_per_block_bytes(int32_t n, const soar_tensor_desc *descs, int32_t *n_groups)
{
    size_t most = 0;
    int32_t groups = 0;
    for (int32_t i = 0; i < n;) {
        const int32_t j = group_end(n, descs, i);
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

size_t batch_workspace_bytes(int32_t n, const soar_tensor_desc *descs)
{
    int32_t groups = 0;
    const size_t most = max_group_per_block_bytes(n, descs, &groups);
    return (groups > 1 ? kLanes : 1) * lane_workspace_bytes(most);
}

hipStream_t aux_stream()
{
    // one per device, created on first use, default priority, never destroyed
    static hipStream_t streams[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    if (!streams[dev]) {
        hipStream_t st = nullptr;
        if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) return nullptr;
        streams[dev] = st;
    }
    return streams[dev];
}

template <int DT>
soar_status launch_group(const Batch &b, uint32_t total_wg, int method, hipStream_t st)
{
    if (b.t[0].amax_in == nullptr) {       // all tensors of a batch supply their maximum, or none does
        ScopedTimer t(SOAR_KERNEL_ABSMAX, st);
        hipLaunchKernelGGL(k_absmax<DT>, dim3(total_wg), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
    }
    if (method == SOAR_METHOD_SOAR) {
        {
            ScopedTimer t(SOAR_KERNEL_STATS, st);
            hipLaunchKernelGGL(k_stats<DT>, dim3(total_wg), dim3(kWG), 0, st, b);
            SOAR_LAUNCH_CHECK();
        }
        ScopedTimer t(SOAR_KERNEL_SEARCH, st);
        hipLaunchKernelGGL((k_search<DT, SOAR_METHOD_SOAR>), dim3(total_wg), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
    } else {
        ScopedTimer t(SOAR_KERNEL_SEARCH, st);
        hipLaunchKernelGGL((k_search<DT, SOAR_METHOD_RTN>), dim3(total_wg), dim3(kWG), 0, st, b);
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
soar_status launch_group_iter(Batch &b, uint32_t total_wg, int iters, hipStream_t st)
{
    {
        ScopedTimer t(SOAR_KERNEL_ABSMAX, st);
        hipLaunchKernelGGL(k_absmax<DT>, dim3(total_wg), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
    }
    {
        ScopedTimer t(SOAR_KERNEL_ITER_INIT, st);
        hipLaunchKernelGGL(k_iter_init<DT>, dim3(total_wg), dim3(kWG), 0, st, b);
        SOAR_LAUNCH_CHECK();
    }
    for (int it = 0; it < iters; ++it) {
        b.iter_t = it;
        ScopedTimer t(SOAR_KERNEL_ITER, st);
        hipLaunchKernelGGL(k_iter<DT>, dim3(total_wg), dim3(kWG), iter_lds_bytes(b), st, b);
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
    if (workspace_bytes < batch_workspace_bytes(n, descs)) return SOAR_ERR_WORKSPACE;

    int32_t n_groups = 0;
    const size_t lane_bytes = lane_workspace_bytes(max_group_per_block_bytes(n, descs, &n_groups));
    const int lanes = (n_groups > 1 && params->streams != 1) ? kLanes : 1;
    char *base = static_cast<char *>(d_workspace);

    hipStream_t lane_stream[kLanes] = {st, st};
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    if (lanes > 1) {
        lane_stream[1] = aux_stream();
        if (!lane_stream[1]) return SOAR_ERR_HIP;
        if (hipEventCreateWithFlags(&ev_fork, hipEventDisableTiming) != hipSuccess) return SOAR_ERR_HIP;
        if (hipEventCreateWithFlags(&ev_join, hipEventDisableTiming) != hipSuccess) {
            (void)hipEventDestroy(ev_fork);
            return SOAR_ERR_HIP;
        }
    }
    soar_status result = SOAR_OK;
    {
        ScopedTimer t(SOAR_KERNEL_INIT, st);
        for (int l = 0; l < lanes && result == SOAR_OK; ++l) {
            hipLaunchKernelGGL(k_init, dim3(kGroupMax * kInitSplit), dim3(kWG), 0, st, base + (size_t)l * lane_bytes);
            if (hipGetLastError() != hipSuccess) result = SOAR_ERR_HIP;
        }
    }
    if (lanes > 1 && result == SOAR_OK) {
        if (hipEventRecord(ev_fork, st) != hipSuccess || hipStreamWaitEvent(lane_stream[1], ev_fork, 0) != hipSuccess)
            result = SOAR_ERR_HIP;
    }
    int32_t g = 0;
    for (int32_t i = 0; i < n && result == SOAR_OK; ++g) {
        const int32_t j = group_end(n, descs, i);
        const int lane = g % lanes;
        char *lane_base = base + (size_t)lane * lane_bytes;
        Batch b;
        std::memset(&b, 0, sizeof(b));
        b.n = (uint32_t)(j - i);
        b.radius = params->dss_radius;
        b.full_search = params->search_mode == SOAR_SEARCH_FULL ? 1 : 0;
        b.n_beta = params->n_beta;
        b.dd_mode = params->dd_mode;
        b.beta_lo = params->beta_lo;
        b.beta_hi = params->beta_hi;
        b.early_stop_rel = params->early_stop_rel;
        b.arm = params->method;
        // the searching iterated kernels are arithmetic-bound: the smallest workgroups balance best
        // (the closed-form arm has no search and streams like the single-step kernels)
        const bool searching = iterated && params->method != SOAR_METHOD_CJSO_ONLY;
        const uint32_t tpw = params->tiles_per_wg ? (uint32_t)params->tiles_per_wg : (searching ? 1u : 0u);
        uint32_t wg = 0;
        char *per_block = lane_base + (size_t)kGroupMax * kSlotBytes;
        for (int32_t k = i; k < j; ++k) {
            const soar_tensor_desc &d = descs[k];
            Task t = make_task(d.d_w, d.rows, d.cols, d.ld_elems, tpw);
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
            result = descs[i].dtype == SOAR_BF16 ? launch_group_iter<SOAR_BF16>(b, wg, params->iters, lane_stream[lane])
                                                 : launch_group_iter<SOAR_FP32>(b, wg, params->iters, lane_stream[lane]);
        else
            result = descs[i].dtype == SOAR_BF16 ? launch_group<SOAR_BF16>(b, wg, params->method, lane_stream[lane])
                                                 : launch_group<SOAR_FP32>(b, wg, params->method, lane_stream[lane]);
        i = j;
    }
    if (lanes > 1) {
        // always join, also after a failed launch, so that the caller's stream stays ordered
        if (hipEventRecord(ev_join, lane_stream[1]) != hipSuccess || hipStreamWaitEvent(st, ev_join, 0) != hipSuccess)
            result = SOAR_ERR_HIP;
        (void)hipEventDestroy(ev_fork);
        (void)hipEventDestroy(ev_join);
    }
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
    return batch_workspace_bytes(n, descs);
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

soar_status soar_quantize_batch(int32_t n, const soar_tensor_desc *descs, const soar_params *params,
                                void *d_workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_batch(n, descs, params, d_workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

soar_status soar_dequantize(const uint8_t *d_codes, const uint8_t *d_scales, const float *d_global_scale,
                            int64_t rows, int64_t cols, soar_dtype out_dtype, void *d_out, int64_t ld_elems,
                            void *hip_stream)
{
    if (!d_codes || !d_scales || !d_global_scale || !d_out) return SOAR_ERR_NULL;
    if (out_dtype != SOAR_BF16 && out_dtype != SOAR_FP32) return SOAR_ERR_DTYPE;
    soar_status s = check_shape(rows, cols, ld_elems);
    if (s != SOAR_OK) return s;
    s = check_matrix_ptr(d_out, out_dtype, ld_elems);
    if (s != SOAR_OK) return s;
    if (reinterpret_cast<uintptr_t>(d_codes) % 8 != 0) return SOAR_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    Task g = make_task(d_out, rows, cols, ld_elems, 0);
    const uint32_t grid = (g.nblk + kWG - 1) / kWG;
    ScopedTimer t(SOAR_KERNEL_DEQUANT, st);
    if (out_dtype == SOAR_BF16)
        hipLaunchKernelGGL(k_dequant<SOAR_BF16>, dim3(grid), dim3(kWG), 0, st, d_codes, d_scales, d_global_scale, g, d_out);
    else
        hipLaunchKernelGGL(k_dequant<SOAR_FP32>, dim3(grid), dim3(kWG), 0, st, d_codes, d_scales, d_global_scale, g, d_out);
    SOAR_LAUNCH_CHECK();
    return SOAR_OK;
}

soar_status soar_recon_error(const void *d_w, soar_dtype dtype, int64_t rows, int64_t cols, int64_t ld_elems,
                             const uint8_t *d_codes, const uint8_t *d_scales, const float *d_global_scale,
                             double *d_sse, void *hip_stream)
{
    if (!d_w || !d_codes || !d_scales || !d_global_scale || !d_sse) return SOAR_ERR_NULL;
    if (dtype != SOAR_BF16 && dtype != SOAR_FP32) return SOAR_ERR_DTYPE;
    soar_status s = check_shape(rows, cols, ld_elems);
    if (s != SOAR_OK) return s;
    s = check_matrix_ptr(d_w, dtype, ld_elems);
    if (s != SOAR_OK) return s;
    if (reinterpret_cast<uintptr_t>(d_codes) % 8 != 0) return SOAR_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    Task g = make_task(d_w, rows, cols, ld_elems, 0);
    uint32_t grid = (g.nblk + kReconWG - 1) / kReconWG;
    if (grid > kReconGrid) grid = kReconGrid;
    ScopedTimer t(SOAR_KERNEL_RECON, st);
    hipLaunchKernelGGL(k_zero_f64, dim3(1), dim3(1), 0, st, d_sse);
    SOAR_LAUNCH_CHECK();
    if (dtype == SOAR_BF16)
        hipLaunchKernelGGL(k_recon<SOAR_BF16>, dim3(grid), dim3(kReconWG), 0, st, g, d_codes, d_scales, d_global_scale, d_sse);
    else
        hipLaunchKernelGGL(k_recon<SOAR_FP32>, dim3(grid), dim3(kReconWG), 0, st, g, d_codes, d_scales, d_global_scale, d_sse);
    SOAR_LAUNCH_CHECK();
    return SOAR_OK;
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
    int32_t j = i + 1;
    while (j < n && j - i < kGroupMax && descs[j].dtype == descs[i].dtype) ++j;
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
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    if (lanes > 1) {
        lane_stream[1] = aux_stream();
        if (!lane_stream[1]) return SOAR_ERR_HIP;
        if (hipEventCreateWithFlags(&ev_fork, hipEventDisableTiming) != hipSuccess) return SOAR_ERR_HIP;
        if (hipEventCreateWithFlags(&ev_join, hipEventDisableTiming) != hipSuccess) {
            (void)hipEventDestroy(ev_fork);
            return SOAR_ERR_HIP;
        }
    }
    soar_status result = SOAR_OK;
    {
        ScopedTimer tm(SOAR_KERNEL_INIT, st);
        hipLaunchKernelGGL(k_init, dim3(lanes * slots * kInitSplit), dim3(kWG), 0, st, base);
        if (hipGetLastError() != hipSuccess) result = SOAR_ERR_HIP;
    }
    if (lanes > 1 && result == SOAR_OK) {
        if (hipEventRecord(ev_fork, st) != hipSuccess || hipStreamWaitEvent(lane_stream[1], ev_fork, 0) != hipSuccess)
            result = SOAR_ERR_HIP;
    }
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
            // the search is arithmetic-bound (smallest workgroups balance best); the plain conversion streams
            uint32_t tpw = params->dss ? 1u : 2u;
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
    if (lanes > 1) {
        // always join, also after a failed launch, so that the caller's stream stays ordered
        if (hipEventRecord(ev_join, lane_stream[1]) != hipSuccess || hipStreamWaitEvent(st, ev_join, 0) != hipSuccess)
            result = SOAR_ERR_HIP;
        (void)hipEventDestroy(ev_fork);
        (void)hipEventDestroy(ev_join);
    }
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

soar_status soar_mxfp4_dequantize(const uint8_t *d_codes, const uint8_t *d_scales, int64_t rows, int64_t cols,
                                  soar_dtype out_dtype, void *d_out, int64_t ld_elems, void *hip_stream)
{
    if (!d_codes || !d_scales || !d_out) return SOAR_ERR_NULL;
    if (out_dtype != SOAR_BF16 && out_dtype != SOAR_FP32) return SOAR_ERR_DTYPE;
    soar_status s = check_mx_shape(rows, cols, ld_elems);
    if (s != SOAR_OK) return s;
    s = check_matrix_ptr(d_out, out_dtype, ld_elems);
    if (s != SOAR_OK) return s;
    if (reinterpret_cast<uintptr_t>(d_codes) % 16 != 0) return SOAR_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const uint32_t nblk = (uint32_t)(rows * (cols / 32));
    const uint32_t grid = (nblk + kWG - 1) / kWG;
    ScopedTimer tm(SOAR_KERNEL_DEQUANT, st);
    if (out_dtype == SOAR_BF16)
        hipLaunchKernelGGL(k_mx_dequant<SOAR_BF16>, dim3(grid), dim3(kWG), 0, st, d_codes, d_scales, nblk,
                           (uint32_t)(cols / 32), ld_elems, ld_elems == cols ? 1u : 0u, d_out);
    else
        hipLaunchKernelGGL(k_mx_dequant<SOAR_FP32>, dim3(grid), dim3(kWG), 0, st, d_codes, d_scales, nblk,
                           (uint32_t)(cols / 32), ld_elems, ld_elems == cols ? 1u : 0u, d_out);
    SOAR_LAUNCH_CHECK();
    return SOAR_OK;
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
    }
    return "unknown status";
}

uint32_t soar_version(void) { return 0x00010000u; }

}  // extern "C"
