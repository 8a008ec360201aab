// Kernels on the stored forms: k_dequant (Eq. 3), k_recon (Eq. 4), k_mx_dequant (MXFP4), and the
// element-wise format kernels the tests use.
#pragma once
#include "soar_device.hpp"
#include "soar_mxfp4.hpp"        // e8m0_value

namespace {


// One stored tensor of a launch: up to kGroupMax tensors share a launch, each with its own range of
// workgroups, so that small tensors do not pay a launch each.
struct StoredTask {
    const uint8_t *codes, *scales;
    const float *gscale;
    const void  *w;          // Eq. 4: the weights
    void        *out;        // Eq. 3: the reconstruction
    double      *sse;        // Eq. 4: the sum
    int64_t  ld;
    uint32_t bpr, nblk, contiguous;
    uint32_t wg_begin, n_wg;
};

struct StoredBatch {
    StoredTask t[kGroupMax];
    uint32_t n;
};

__device__ __forceinline__ uint32_t find_task(const StoredBatch &b, uint32_t &lwg)
{
    const uint32_t id = blockIdx.x;
    uint32_t k = 0;
    for (uint32_t j = 1; j < b.n; ++j)
        if (id >= b.t[j].wg_begin) k = j;
    lwg = id - b.t[k].wg_begin;
    return k;
}

// Eq. 3
template <int DT>
__global__ __launch_bounds__(kWG) void k_dequant(const StoredBatch batch)
{
    constexpr int kP = pieces_per_block<DT, 16>();
    __shared__ u32x4 s_x[kWG * kP];                    // store_wave_blocks: one region per wave
    uint32_t lwg;
    const StoredTask g = batch.t[find_task(batch, lwg)];
    const uint32_t i = lwg * kWG + threadIdx.x;
    const uint32_t wave_first = i - (threadIdx.x & 63u);
    if (wave_first >= g.nblk) return;
    float v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = 0.0f;
    if (i < g.nblk) {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        const float s = *g.gscale * e4m3_value(__builtin_nontemporal_load(g.scales + i));
        const u32x2 nb = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(g.codes) + i);
        float q[16];
        fp4x8_values(nb.x, q);
        fp4x8_values(nb.y, q + 8);
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = q[j] * s;
    }
    if (g.contiguous) {
        // packed rows: the wave writes its 64 blocks in coalesced pieces (all of its lanes take part)
        store_wave_blocks<DT, 16>(g.out, wave_first, g.nblk, s_x + (threadIdx.x >> 6) * (64 * kP), v);
        return;
    }
    if (i >= g.nblk) return;
    const size_t off = block_offset(g.contiguous != 0u, g.bpr, g.ld, i);
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
        uint4 *p = reinterpret_cast<uint4 *>(static_cast<uint16_t *>(g.out) + off);
        p[0] = make_uint4(u[0], u[1], u[2], u[3]);
        p[1] = make_uint4(u[4], u[5], u[6], u[7]);
    } else {
        float4 *p = reinterpret_cast<float4 *>(static_cast<float *>(g.out) + off);
#pragma unroll
        for (int k = 0; k < 4; ++k) p[k] = make_float4(v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]);
    }
}

// MXFP4: w^ = q * 2^(e-127) per block of 32 (bpr counts blocks of 32; gscale is unused)
template <int DT>
__global__ __launch_bounds__(kWG) void k_mx_dequant(const StoredBatch batch)
{
    constexpr int kP = pieces_per_block<DT, 32>();
    __shared__ u32x4 s_x[kWG * kP];                    // store_wave_blocks: one region per wave
    uint32_t lwg;
    const StoredTask g = batch.t[find_task(batch, lwg)];
    const uint8_t *codes = g.codes, *scales = g.scales;
    const uint32_t nblk = g.nblk, bpr = g.bpr, contiguous = g.contiguous;
    const int64_t ld = g.ld;
    void *out = g.out;
    const uint32_t i = lwg * kWG + threadIdx.x;
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

// clears the sums of a call of k_recon launches (a kernel, not a memset: the call may be captured into a graph);
// one launch for up to kZeroMax tensors, whose addresses travel in the kernel arguments
constexpr int kZeroMax = 448;
struct ZeroBatch {
    double *sum[kZeroMax];
    uint32_t n;
};
static_assert(sizeof(ZeroBatch) <= 4096, "kernel arguments");
__global__ __launch_bounds__(kZeroMax) void k_zero_sums(const ZeroBatch batch)
{
    if (threadIdx.x < batch.n) *batch.sum[threadIdx.x] = 0.0;
}

// Eq. 4 for stored codes and scales.  Every workgroup ends with one binary64 atomic addition to its
// tensor's result; additions to one address are served one after the other (thousands of them cost
// more than the reads of a whole tensor), so the workgroups are few and large: 16 waves each, at most
// kReconGrid per tensor.
constexpr int kReconWG = 1024;
constexpr uint32_t kReconGrid = 256;      // 512: 5 % slower on the full-model workload, 8 % on 448 MiB tensors; 64-128: as 256
template <int DT>
__global__ __launch_bounds__(kReconWG) void k_recon(const StoredBatch batch)
{
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    constexpr int kP = pieces_per_block<DT, 16>();
    __shared__ u32x4 s_x[kReconWG * kP];               // load_wave_blocks: one region per wave
    __shared__ double s_wave[kReconWG / 64];
    uint32_t lwg;
    const StoredTask g = batch.t[find_task(batch, lwg)];
    const uint32_t tid = threadIdx.x;
    const float alpha = *g.gscale;
    double sse = 0.0;
    // the workgroups of a tensor sweep one contiguous window of memory
    for (uint32_t first = lwg * kReconWG; first < g.nblk; first += g.n_wg * kReconWG) {
        const uint32_t i = first + tid;
        const bool inside = i < g.nblk;
        float w[16], q[16];
        if (g.contiguous) load_wave_blocks<DT, 16, true>(g.w, i - (tid & 63u), g.nblk, s_x + (tid >> 6) * (64 * kP), w);
        else if (inside) load_block<DT, false>(g.w, block_offset(false, g.bpr, g.ld, i), w);
        if (inside) {
            const u32x2 nb = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(g.codes) + i);
            fp4x8_values(nb.x, q);
            fp4x8_values(nb.y, q + 8);
            sse += (double)block_error(w, q, alpha * e4m3_value(__builtin_nontemporal_load(g.scales + i)));
        }
    }
    sse = wave_pair_tree(sse);
    if ((tid & 63) == 0) s_wave[tid >> 6] = sse;
    __syncthreads();
    if (tid < 64) {
        double v = tid < kReconWG / 64 ? s_wave[tid] : 0.0;
        v = wave_pair_tree(v);
        if (tid == 0) atomicAdd(g.sse, v);
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

}  // namespace
