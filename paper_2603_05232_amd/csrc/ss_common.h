// Shared host/device helpers of the SlideSparse gfx950 library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "slidesparse.h"

#define SS_FORMAT_VERSION 2

namespace ss {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v16bf __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v16h __attribute__((ext_vector_type(16)));

// Rows of the packed weight buffers are padded to this many output channels; one such
// panel is the O-extent a wave accumulates, and the row order inside a panel is permuted
// so that every lane ends up holding runs of consecutive output channels.
constexpr int PANEL = 128;
// K' granularity of the packed format and of both GEMMs.
constexpr int KSTEP = 128;

// Alg. 1: n_g = ceil(K / 2N) blocks (the last one completed with zeros), K' = 4 n_g (N-1).
__host__ __device__ inline int64_t n_groups(int64_t K, int N) { return (K + 2 * N - 1) / (2 * N); }
__host__ __device__ inline int64_t lifted_k(int64_t K, int N) { return n_groups(K, N) * 4 * (N - 1); }
// Stored width (elements of es bytes) of a lifted row: K' rounded up to whole 128-byte k units;
// the columns beyond K' hold zeros (activations) / all-zero windows (weights).
inline int64_t lifted_ld(int64_t K, int N, int es) { const int64_t per = KSTEP / es; return (lifted_k(K, N) + per - 1) / per * per; }
inline bool valid_N(int N) { return N >= 2 && N <= 8; }
inline int elem_size(ss_dtype d) { return (d == SS_BF16 || d == SS_FP16) ? 2 : 1; }
inline bool valid_dtype(ss_dtype d) { return d == SS_I8 || d == SS_FP8_E4M3 || d == SS_BF16 || d == SS_FP16; }
inline bool unscaled(ss_dtype d) { return d == SS_BF16 || d == SS_FP16; }
inline ss_status launch_status()
{
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

// ---- scalar format conversions (device) --------------------------------------------------
__device__ inline float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ inline uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// fp32 -> IEEE half bits, round to nearest even (v_cvt_f16_f32)
__device__ inline uint16_t f32_to_f16_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

// fp32 (already clamped to [-448, 448]) -> OCP e4m3fn byte, round to nearest even.
__device__ inline uint32_t f32_to_e4m3(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t sign = (u >> 24) & 0x80u;
    float a = __uint_as_float(u & 0x7FFFFFFFu);
    uint32_t code;
    if (a < 0.015625f) {                       // below 2^-6: multiples of 2^-9
        code = (uint32_t)rintf(a * 512.0f);    // 0..8; 8 is the smallest normal
    } else {
        uint32_t m = __float_as_uint(a);
        m += 0x7FFFFu + ((m >> 20) & 1u);      // rne to 3 mantissa bits, may carry into the exponent
        code = (m >> 20) - ((127u - 7u) << 3);
        code = code > 0x7Eu ? 0x7Eu : code;
    }
    return sign | code;
}

}  // namespace ss
