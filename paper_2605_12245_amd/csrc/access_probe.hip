// HBM access patterns of the block-per-lane kernels, on gfx950: what a lane's own 32, 64 or 128
// contiguous bytes cost against fully coalesced 16-byte pieces, with ordinary and with streaming
// (nontemporal) accesses, and what the wave-private LDS exchange recovers.
//
// Read cases: a read-only kernel over 434 MiB (one MXFP4 launch group of the full-model workload),
// optionally with the stores of a quantizer (1/4 of the bytes as codes, one byte per block).
// Write cases: a decode-and-expand kernel (8 bytes of codes and one scale byte in, 32 or 64 bytes
// out per lane: the shape of dequantization to bf16 / fp32).
// No arithmetic of the method: the values are irrelevant.  Every size is a multiple of a tile.
//
// Build: hipcc --offload-arch=gfx950 -O3 access_probe.hip -o access_probe     Run: ./access_probe
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                       \
    do {                                                               \
        if ((x) != hipSuccess) {                                       \
            std::printf("HIP error at line %d\n", __LINE__);           \
            return 1;                                                  \
        }                                                              \
    } while (0)

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
constexpr int kWG = 256;

// slot of piece `piece` of unit `unit` in a wave's LDS region: rotated by the unit's row of 256 bytes
template <int P>
__device__ __forceinline__ uint32_t slot(uint32_t unit, uint32_t piece)
{
    return unit * P + ((piece + unit / (16 / P)) & (P - 1));
}

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// P pieces of 16 bytes per lane.  EXCHANGE: coalesced pieces, then through LDS to the owning lane.
// NT: nontemporal loads.  WRITE: also store 4 P bytes and one byte per lane, nontemporal.
template <int P, bool EXCHANGE, bool NT, bool WRITE>
__global__ __launch_bounds__(kWG) void k_read(const u32x4 *in, uint32_t *out, uint8_t *out2, uint32_t units, uint32_t *sink)
{
    __shared__ u32x4 s_x[EXCHANGE ? kWG * P : 1];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t i = blockIdx.x * kWG + tid;
    if (i >= units) return;
    u32x4 v[P];
    if constexpr (EXCHANGE) {
        const u32x4 *range = in + (size_t)(i - lane) * P;
        u32x4 *sw = s_x + wave * 64 * P;
#pragma unroll
        for (int p = 0; p < P; ++p) v[p] = NT ? __builtin_nontemporal_load(range + p * 64 + lane) : range[p * 64 + lane];
#pragma unroll
        for (int p = 0; p < P; ++p) sw[slot<P>((p * 64 + lane) / P, (p * 64 + lane) % P)] = v[p];
        wave_sync();
#pragma unroll
        for (int p = 0; p < P; ++p) v[p] = sw[slot<P>(lane, p)];
    } else {
#pragma unroll
        for (int p = 0; p < P; ++p) v[p] = NT ? __builtin_nontemporal_load(in + (size_t)i * P + p) : in[(size_t)i * P + p];
    }
    uint32_t a = 0;
#pragma unroll
    for (int p = 0; p < P; ++p) a ^= v[p].x ^ v[p].y ^ v[p].z ^ v[p].w;
    if constexpr (WRITE) {
#pragma unroll
        for (int p = 0; p < P; ++p) __builtin_nontemporal_store(a + p, out + (size_t)i * P + p);
        __builtin_nontemporal_store((uint8_t)a, out2 + i);
    }
    if (a == 0x12345678u) sink[0] = a;       // keeps the loads alive
}

// MODE 0: the lane's own P pieces, ordinary stores; 1: the same, nontemporal; 2: coalesced through LDS,
// nontemporal; 3: coalesced through LDS, ordinary
template <int P, int MODE>
__global__ __launch_bounds__(kWG) void k_expand(const u32x2 *codes, const uint8_t *scales, u32x4 *out, uint32_t units)
{
    __shared__ u32x4 s_x[MODE >= 2 ? kWG * P : 1];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t i = blockIdx.x * kWG + tid;
    if (i >= units) return;
    const u32x2 c = __builtin_nontemporal_load(codes + i);
    const uint32_t sc = __builtin_nontemporal_load(scales + i);
    u32x4 v[P];
#pragma unroll
    for (int p = 0; p < P; ++p) v[p] = u32x4{c.x + sc + p, c.y ^ sc, c.x * 3u + p, c.y + 7u};
    if constexpr (MODE < 2) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if constexpr (MODE == 1) __builtin_nontemporal_store(v[p], out + (size_t)i * P + p);
            else out[(size_t)i * P + p] = v[p];
        }
    } else {
        u32x4 *sw = s_x + wave * 64 * P;
        u32x4 *range = out + (size_t)(i - lane) * P;
#pragma unroll
        for (int p = 0; p < P; ++p) sw[slot<P>(lane, p)] = v[p];
        wave_sync();
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const u32x4 x = sw[slot<P>((p * 64 + lane) / P, (p * 64 + lane) % P)];
            if constexpr (MODE == 2) __builtin_nontemporal_store(x, range + p * 64 + lane);
            else range[p * 64 + lane] = x;
        }
    }
}

struct Buffers {
    u32x4 *in = nullptr, *out = nullptr;
    uint8_t *small = nullptr;
    uint32_t *sink = nullptr;
};

template <typename Launch>
int timed(const char *name, double bytes_main, double bytes_all, Launch launch)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int r = 0; r < 3; ++r) launch();
    CHECK(hipDeviceSynchronize());
    const int reps = 20;
    CHECK(hipEventRecord(e0, 0));
    for (int r = 0; r < reps; ++r) launch();
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.0f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double per = ms / reps * 1e-3;
    std::printf("  %-52s %7.1f us  %5.2f TB/s (%5.2f TB/s of all traffic)\n", name, per * 1e6, bytes_main / per / 1e12,
                bytes_all / per / 1e12);
    std::fflush(stdout);
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return 0;
}

template <int P, bool EXCHANGE, bool NT, bool WRITE>
int read_case(const char *name, const Buffers &b, size_t bytes)
{
    const uint32_t units = (uint32_t)(bytes / (16 * P));
    const double all = (double)bytes * (WRITE ? 1.25 + 1.0 / (16 * P) : 1.0);
    return timed(name, (double)bytes, all, [&] {
        hipLaunchKernelGGL((k_read<P, EXCHANGE, NT, WRITE>), dim3(units / kWG), dim3(kWG), 0, 0, b.in,
                           reinterpret_cast<uint32_t *>(b.out), b.small, units, b.sink);
    });
}

template <int P, int MODE>
int write_case(const char *name, const Buffers &b, uint32_t units)
{
    return timed(name, (double)units * 16 * P, (double)units * (9.0 + 16.0 * P), [&] {
        hipLaunchKernelGGL((k_expand<P, MODE>), dim3(units / kWG), dim3(kWG), 0, 0, reinterpret_cast<const u32x2 *>(b.in),
                           b.small, b.out, units);
    });
}

}  // namespace

int main(int argc, char **argv)
{
    // optional argument: MiB read per launch (default 434; a multiple of 32 KiB); beyond the 256 MiB last-level
    // cache plus what one repetition leaves behind, every read comes from HBM
    const size_t read_bytes = (size_t)(argc > 1 ? atol(argv[1]) : 434) << 20;
    const uint32_t write_units = 12u << 20;           // blocks of 16 weights: 384 MiB of bf16 out, 768 MiB of fp32
    if (read_bytes == 0 || read_bytes % ((size_t)kWG * 128) != 0 || read_bytes > ((size_t)8 << 30)) {
        std::printf("size: a multiple of 32 KiB, at most 8 GiB\n");
        return 1;
    }
    // the read cases with stores write read_bytes / 4 of `out` and read_bytes / 32 of `small`;
    // the write cases write write_units * 64 of `out` and read write_units of `small` and 8 * write_units of `in`
    const size_t out_bytes = read_bytes / 4 > (size_t)write_units * 64 ? read_bytes / 4 : (size_t)write_units * 64;
    const size_t small_bytes = read_bytes / 32 > write_units ? read_bytes / 32 : write_units;
    if (read_bytes < (size_t)write_units * 8) {
        std::printf("size: at least %zu MiB\n", ((size_t)write_units * 8) >> 20);
        return 1;
    }
    Buffers b;
    CHECK(hipMalloc(&b.in, read_bytes));
    CHECK(hipMalloc(&b.out, out_bytes));
    CHECK(hipMalloc(&b.small, small_bytes));
    CHECK(hipMalloc(&b.sink, 4));
    CHECK(hipMemset(b.in, 1, read_bytes));
    CHECK(hipMemset(b.small, 2, write_units));

    std::printf("reads of %zu MiB (TB/s of reads)\n", read_bytes >> 20);
    if (read_case<1, false, true, false>("16 B per lane (coalesced), streaming", b, read_bytes)) return 1;
    if (read_case<1, false, false, false>("16 B per lane (coalesced), ordinary", b, read_bytes)) return 1;
    if (read_case<2, false, true, false>("32 B per lane, streaming", b, read_bytes)) return 1;
    if (read_case<2, false, false, false>("32 B per lane, ordinary", b, read_bytes)) return 1;
    if (read_case<2, true, true, false>("32 B per lane through the exchange, streaming", b, read_bytes)) return 1;
    if (read_case<4, false, true, false>("64 B per lane, streaming", b, read_bytes)) return 1;
    if (read_case<4, false, false, false>("64 B per lane, ordinary", b, read_bytes)) return 1;
    if (read_case<4, true, true, false>("64 B per lane through the exchange, streaming", b, read_bytes)) return 1;
    if (read_case<4, true, false, false>("64 B per lane through the exchange, ordinary", b, read_bytes)) return 1;
    std::printf("the same reads with a quantizer's stores (1/4 of the bytes + 1 byte per lane)\n");
    if (read_case<2, false, true, true>("32 B per lane, streaming", b, read_bytes)) return 1;
    if (read_case<2, true, true, true>("32 B per lane through the exchange, streaming", b, read_bytes)) return 1;
    if (read_case<4, false, true, true>("64 B per lane, streaming", b, read_bytes)) return 1;
    if (read_case<4, false, false, true>("64 B per lane, ordinary", b, read_bytes)) return 1;
    if (read_case<4, true, true, true>("64 B per lane through the exchange, streaming", b, read_bytes)) return 1;
    std::printf("writes of a decode-and-expand kernel, %u lanes (TB/s written)\n", write_units);
    if (write_case<2, 0>("32 B per lane (bf16 out), ordinary", b, write_units)) return 1;
    if (write_case<2, 1>("32 B per lane (bf16 out), streaming", b, write_units)) return 1;
    if (write_case<2, 2>("32 B per lane through the exchange, streaming", b, write_units)) return 1;
    if (write_case<2, 3>("32 B per lane through the exchange, ordinary", b, write_units)) return 1;
    if (write_case<4, 0>("64 B per lane (fp32 out), ordinary", b, write_units)) return 1;
    if (write_case<4, 1>("64 B per lane (fp32 out), streaming", b, write_units)) return 1;
    if (write_case<4, 2>("64 B per lane through the exchange, streaming", b, write_units)) return 1;
    if (write_case<4, 3>("64 B per lane through the exchange, ordinary", b, write_units)) return 1;
    return 0;
}
