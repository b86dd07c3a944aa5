// Shared host-side plumbing of libtma: error reporting, argument checks,
// launch helpers.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "tma.h"

namespace tma {

constexpr int kWave = 64;  // CDNA wavefront width

// Thread-local message returned by tma_last_error().
char *error_buffer();
int fail(int code, const char *fmt, ...);

inline hipStream_t as_stream(tma_stream_t s) { return reinterpret_cast<hipStream_t>(s); }

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Checks the launch itself (bad configuration, missing code object); kernel
// execution errors surface at the caller's next synchronisation.
inline int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TMA_ERR_HIP, "%s: launch failed: %s", what, hipGetErrorString(e));
    return TMA_OK;
}

// Optional per-kernel timing with HIP events recorded on the launch stream
// (tma_profile_begin / tma_profile_end).  Costs nothing while disabled.
class KernelTimer {
public:
    KernelTimer(const char *name, hipStream_t stream);
    ~KernelTimer();
    KernelTimer(const KernelTimer &) = delete;
    KernelTimer &operator=(const KernelTimer &) = delete;

private:
    int slot_;
    hipStream_t stream_;
};
#define TMA_TIMED(name, stream) ::tma::KernelTimer tma_kernel_timer_(name, stream)

#define TMA_HIP_TRY(expr, what)                                                          \
    do {                                                                                 \
        hipError_t e_ = (expr);                                                          \
        if (e_ != hipSuccess)                                                            \
            return ::tma::fail(TMA_ERR_HIP, "%s: %s", what, hipGetErrorString(e_));      \
    } while (0)

#define TMA_REQUIRE(cond, code, ...)                                                     \
    do {                                                                                 \
        if (!(cond)) return ::tma::fail(code, __VA_ARGS__);                              \
    } while (0)

// bf16 <-> fp32, round-to-nearest-even on store (NaN kept quiet).
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}

// Output number (unit+1) of the SplitMix64 stream (Steele, Lea, Flood 2014) seeded with `seed`: the library's
// counter-based generator (partition assignment, mini-batch draws).
__host__ __device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t unit)
{
    uint64_t z = seed + (unit + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// A 16-byte piece of a feature row: 4 fp32 or 8 bf16 elements, handled as fp32 in registers.
template <typename T>
struct Chunk;

template <>
struct Chunk<float> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void load(const float *p, float (&v)[4])
    {
        const float4 x = *reinterpret_cast<const float4 *>(p);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    }
    static __device__ __forceinline__ void widen(const uint4 &x, float (&v)[4])
    {
        v[0] = __uint_as_float(x.x); v[1] = __uint_as_float(x.y); v[2] = __uint_as_float(x.z); v[3] = __uint_as_float(x.w);
    }
    static __device__ __forceinline__ void store(float *p, const float (&v)[4])
    {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};

template <>
struct Chunk<uint16_t> {  // bf16 storage
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void load(const uint16_t *p, float (&v)[8])
    {
        widen(*reinterpret_cast<const uint4 *>(p), v);
    }
    static __device__ __forceinline__ void widen(const uint4 &x, float (&v)[8])
    {
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ void store(uint16_t *p, const float (&v)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = uint32_t(f32_to_bf16(v[2 * i])) | (uint32_t(f32_to_bf16(v[2 * i + 1])) << 16);
        *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

}  // namespace tma
