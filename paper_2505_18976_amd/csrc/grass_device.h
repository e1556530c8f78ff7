// Shared device/host helpers of the GraSS kernels: the counter hash, status
// plumbing and small launch utilities.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "grass.h"

namespace grass {

// splitmix64 (Steele, Lea, Flood 2014).  The paper only says that indices and
// signs are sampled (App. B.4.1); every random choice here is the c-th output
// of the generator seeded with a per-role sub-seed, computed in registers.
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;

__host__ __device__ __forceinline__ uint64_t finalise(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// c-th output (0-based) of the generator seeded with `seed`.
__host__ __device__ __forceinline__ uint64_t sm(uint64_t seed, uint64_t c) {
    return finalise(seed + (c + 1) * kGamma);
}

// Sub-seed of a stream: H(seed, stream, c) = sm(substream(seed, stream), c).
inline uint64_t substream(uint64_t seed, uint64_t stream_id) { return sm(seed, stream_id); }

// Bucket inside a block of m rows and sign bit (already shifted to bit 31)
// from one hash value (Sec. 3.1: each input coordinate picks its output
// coordinates and whether to add or subtract).
__device__ __forceinline__ uint32_t bucket_of(uint64_t h, uint32_t m) {
    return __umulhi((uint32_t)(h >> 32), m);
}
__device__ __forceinline__ uint32_t signbit_of(uint64_t h) { return ((uint32_t)h & 1u) << 31; }

inline hipStream_t as_stream(grass_stream s) { return reinterpret_cast<hipStream_t>(s); }

inline grass_status launch_status() {
    return hipGetLastError() == hipSuccess ? GRASS_OK : GRASS_EHIP;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// out[i, b] = scale * sum_c partial[c][i][b] with c ascending: the fixed-order
// cross-workgroup reduction used instead of global floating-point atomics.
static __global__ void __launch_bounds__(256) reduce_partials_kernel(const float* partial, uint64_t n, uint32_t k,
                                                                     uint32_t chunks, float scale, float* out,
                                                                     uint64_t ldo) {
    const uint64_t total = n * k;
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const uint64_t i = t / k;
    const uint32_t b = (uint32_t)(t - i * k);
    float sum = 0.0f;
    for (uint32_t c = 0; c < chunks; ++c) sum += partial[(uint64_t)c * total + t];
    out[i * ldo + b] = sum * scale;
}

// dst (k x ld_dst) = transpose of rows [r0, r0+rc) of src (N x k); columns rc..rc_pad of dst are zero-filled.
static __global__ void __launch_bounds__(256) transpose_rows_kernel(const float* src, uint64_t ld_src, uint64_t r0, uint32_t rc,
                                                            uint32_t rc_pad, uint32_t k, float* dst, uint64_t ld_dst) {
    __shared__ float tile[64][65];
    const uint32_t c0 = blockIdx.x * 64;      // column of src = row of dst
    const uint32_t q0 = blockIdx.y * 64;      // row of the chunk = column of dst
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const uint32_t q = q0 + r, c = c0 + tx;
        tile[r][tx] = (q < rc && c < k) ? src[(r0 + q) * ld_src + c] : 0.0f;
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const uint32_t c = c0 + r, q = q0 + tx;
        if (c < k && q < rc_pad) dst[(uint64_t)c * ld_dst + q] = tile[tx][r];
    }
}

constexpr int kNumCU = 256;                 // MI355X
constexpr size_t kLdsBytes = 160 * 1024;    // per CU and per workgroup on gfx950

// A kernel that uses more than 64 KB of dynamic LDS has to be allowed to, once per device (the setting belongs to
// the device's copy of the code object).  One LdsOptIn per kernel remembers the devices that have it; the flags are
// atomic so that host threads may call the library concurrently (two threads that race on a fresh device both set
// the attribute, which is harmless).
struct LdsOptIn { std::atomic<bool> done[64] = {}; };
inline hipError_t allow_large_lds(LdsOptIn& state, const void* kernel) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && state.done[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
    if (e == hipSuccess && tracked) state.done[dev].store(true, std::memory_order_release);
    return e;
}

}  // namespace grass
