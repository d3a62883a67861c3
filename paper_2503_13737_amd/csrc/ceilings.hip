// Measurement aid: micro-kernels that show what this machine reaches for the access and
// instruction patterns the attention kernels are built from -- a streaming read with the
// non-temporal hint, reads of randomly placed contiguous chunks (the pattern of a paged cache: one
// (page, head) tile of 16 tokens is 4 KiB), and matrix instructions issued back to back from
// registers.  bench.py times them next to the real kernels and reports the kernels' rates as a
// fraction of these ceilings as well as of the published peaks.  None of them touches the caller's
// data beyond reading `buf`.
#include <hip/hip_runtime.h>

#include "../../include/mpa.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWgs = 4096;        // work-groups of the read kernels (256 threads each)
constexpr int kMfmaWgs = 1024;    // two work-groups per compute unit, one wavefront per SIMD each

// Every lane of the chip reads 16 bytes per load, eight loads in flight per lane, over the whole
// buffer once.
__global__ void __launch_bounds__(256)
stream_read_kernel(const u32x4 *__restrict__ p, size_t n_vec, uint32_t *sink)
{
    constexpr int U = 8;
    size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256 * U;
    uint32_t acc = 0;
    for (; i + (U - 1) * 256 < n_vec; i += stride) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u) sink[0] = acc;   // keeps the loads alive; practically never true
}

__device__ __forceinline__ uint64_t mix(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// One wavefront reads `chunks_per_wave` chunks of LOADS KiB each at pseudo-random chunk positions,
// two chunks in flight (what a generation row does with the pages of its sequence).
template <int LOADS>
__global__ void __launch_bounds__(256)
random_chunk_kernel(const u32x4 *__restrict__ p, uint64_t n_chunks, int32_t chunks_per_wave, uint32_t *sink)
{
    const int lane = threadIdx.x & 63;
    const uint64_t wave = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    uint32_t acc = 0;
    u32x4 a[LOADS], b[LOADS];
    auto issue = [&](u32x4 (&r)[LOADS], int32_t c) {
        const uint64_t chunk = mix(wave * 1000003ull + (uint64_t)c) % n_chunks;
        const u32x4 *src = p + chunk * (LOADS * 64) + lane;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) r[i] = __builtin_nontemporal_load(src + i * 64);
    };
    auto use = [&](u32x4 (&r)[LOADS]) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) acc ^= r[i].x ^ r[i].y ^ r[i].z ^ r[i].w;
    };
    issue(a, 0);
    for (int32_t c = 0; c < chunks_per_wave; c += 2) {
        issue(b, c + 1);
        use(a);
        issue(a, c + 2);
        use(b);
    }
    use(a);
    if (acc == 0x12345678u) sink[0] = acc;
}

// Four independent accumulators per wavefront, `iters` rounds of four 32x32x16 bf16 products.
// Operands: a smooth pattern with few mantissa bits set, or (noisy) pseudo-random values of unit
// scale with full mantissas, like the q/K/V of the benchmark batches -- the second kind makes the
// matrix pipe draw more power, and the clock the chip sustains under it is lower.
__global__ void __launch_bounds__(256)
mfma_loop_kernel(float *sink, int32_t iters, int32_t noisy)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(threadIdx.x * 0.001f + i);
        b[i] = (__bf16)(i * 0.5f);
    }
    if (noisy) {
        for (int i = 0; i < 8; ++i) {
            const uint64_t r = mix(((uint64_t)blockIdx.x * 256 + threadIdx.x) * 8 + i);
            // two uniforms in (-1, 1) with 23 random bits each, summed: unit-scale, full mantissa after rounding
            const float u = (float)(int32_t)(r & 0xFFFFFF) * (1.f / 8388608.f) - 1.f;
            const float v = (float)(int32_t)((r >> 24) & 0xFFFFFF) * (1.f / 8388608.f) - 1.f;
            a[i] = (__bf16)(u + v);
            b[i] = (__bf16)(u - v);
        }
    }
    f32x16 c[4];
    for (int k = 0; k < 4; ++k)
        for (int i = 0; i < 16; ++i) c[k][i] = 0.f;
    for (int32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 4; ++k) c[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[k], 0, 0, 0);
    }
    float s = 0.f;
    for (int k = 0; k < 4; ++k)
        for (int i = 0; i < 16; ++i) s += c[k][i];
    if (s == 12345.678f) sink[0] = s;
}

}  // namespace

extern "C" int64_t mpa_ceiling_launch(int32_t kind, const void *buf, size_t bytes, int32_t iters, void *sink, void *stream)
{
    if (!sink || (reinterpret_cast<uintptr_t>(sink) % 4) != 0) return MPA_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    int64_t work = 0;
    switch (kind) {
    case MPA_CEIL_STREAM_READ: {
        if (!buf || (reinterpret_cast<uintptr_t>(buf) % 16) != 0 || bytes < ((size_t)1 << 20)) return MPA_ERR_INVALID_ARG;
        const size_t per_pass = (size_t)kWgs * 256 * 8 * 16;     // whole passes of the grid only
        const size_t n_vec = bytes / per_pass * per_pass / 16;
        if (n_vec == 0) return MPA_ERR_INVALID_ARG;
        hipLaunchKernelGGL(stream_read_kernel, dim3(kWgs), dim3(256), 0, s, (const u32x4 *)buf, n_vec, (uint32_t *)sink);
        work = (int64_t)n_vec * 16;
        break;
    }
    case MPA_CEIL_RANDOM_4K:
    case MPA_CEIL_RANDOM_16K: {
        const int kib = kind == MPA_CEIL_RANDOM_4K ? 4 : 16;
        if (!buf || (reinterpret_cast<uintptr_t>(buf) % 16) != 0 || iters < 2 || iters % 2 != 0) return MPA_ERR_INVALID_ARG;
        if (bytes < (size_t)kib * 1024 * 64) return MPA_ERR_INVALID_ARG;
        const uint64_t n_chunks = bytes / ((size_t)kib * 1024);
        if (kib == 4)
            hipLaunchKernelGGL(random_chunk_kernel<4>, dim3(kWgs), dim3(256), 0, s, (const u32x4 *)buf, n_chunks, iters, (uint32_t *)sink);
        else
            hipLaunchKernelGGL(random_chunk_kernel<16>, dim3(kWgs), dim3(256), 0, s, (const u32x4 *)buf, n_chunks, iters, (uint32_t *)sink);
        work = (int64_t)kWgs * 4 * ((int64_t)iters + 1) * kib * 1024;   // chunks 0 .. iters are read
        break;
    }
    case MPA_CEIL_MFMA_BF16:
    case MPA_CEIL_MFMA_BF16_NOISY: {
        if (iters < 1) return MPA_ERR_INVALID_ARG;
        hipLaunchKernelGGL(mfma_loop_kernel, dim3(kMfmaWgs), dim3(256), 0, s, (float *)sink, iters,
                           kind == MPA_CEIL_MFMA_BF16_NOISY ? 1 : 0);
        work = (int64_t)kMfmaWgs * 4 * (int64_t)iters * 4 * (2ll * 32 * 32 * 16);
        break;
    }
    default: return MPA_ERR_INVALID_ARG;
    }
    return hipGetLastError() == hipSuccess ? work : (int64_t)MPA_ERR_HIP;
}
