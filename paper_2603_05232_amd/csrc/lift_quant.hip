// act_lift_quant: fused per-token quantisation + activation lifting (Alg. 1), and
// slide_prune_quant: offline (2N-2):2N magnitude pruning + per-channel quantisation.
//
// Both kernels stream a row through one workgroup: the row is read from HBM once, kept in
// registers while the wavefronts reduce the absmax, quantised element-wise into LDS, and the
// lifted windows are then gathered from LDS so that every source element is quantised once
// and every output store is a coalesced 16-byte vector.  HBM traffic per token is therefore
// the algorithmic minimum: K input elements in, K' output elements + one scale out.
#include "ss_common.h"

namespace ss {

constexpr int LQ_THREADS = 256;

template <typename T> struct InVec;
template <> struct InVec<float> {
    static constexpr int N = 4; typedef float4 V;
    __device__ static void unpack(const V& v, float* f) { f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w; }
};
template <> struct InVec<uint16_t> {          // bf16 bits
    static constexpr int N = 8; typedef uint4 V;
    __device__ static void unpack(const V& v, float* f)
    {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    }
};
__device__ inline float load_scalar(const float* p) { return *p; }
__device__ inline float load_scalar(const uint16_t* p) { return bf16_bits_to_f32(*p); }

template <int THREADS> __device__ inline float block_absmax(float v, float* red)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float m = red[0];
#pragma unroll
    for (int w = 1; w < THREADS / 64; ++w) m = fmaxf(m, red[w]);
    return m;
}

// quantise one element: OUT 0 = int8, 1 = fp8 e4m3, 2 = bf16 (no scale), 3 = half (no scale)
template <int OUT> __device__ inline uint32_t quant1(float x, float r)
{
    if constexpr (OUT == 0) {
        float q = rintf(x * r);
        q = fminf(fmaxf(q, -127.0f), 127.0f);
        return (uint32_t)(int)q & 0xFFu;
    } else if constexpr (OUT == 1) {
        float q = x * r;
        q = fminf(fmaxf(q, -448.0f), 448.0f);
        return f32_to_e4m3(q);
    } else if constexpr (OUT == 2) {
        return f32_to_bf16_bits(x);
    } else {
        return f32_to_f16_bits(x);
    }
}

// MAXV > 0: vector loads, row kept in registers (needs K <= MAXV * THREADS * VecN, 16-byte
// aligned rows).  MAXV == 0: scalar loads, second pass re-reads the row.  Long rows take more
// threads per token rather than more registers per thread: the loads of a token are all in
// flight at once either way, but fewer registers leave room for more tokens per compute unit.
template <typename TIN, int OUT, int MAXV, int THREADS>
__global__ __launch_bounds__(THREADS) void k_act_lift_quant(const TIN* __restrict__ X, int64_t ldx, int K, int N,
                                                                uint8_t* __restrict__ XL, float* __restrict__ s_x, int Kp, int Kz)
{
    // Kp: stored width of a lifted row (whole 128-byte units); Kz >= n_g * 2N + 8 / ES: elements
    // of the quantised row held in LDS, those at and beyond K being zero (zero-completed last block)
    constexpr int ES = OUT >= 2 ? 2 : 1;                 // output element bytes
    extern __shared__ uint32_t lds[];                     // Kz * ES bytes
    __shared__ float red[THREADS / 64];
    const int64_t m = blockIdx.x;
    const TIN* x = X + m * ldx;
    const int t = threadIdx.x;
    typedef InVec<TIN> IV;
    typename IV::V v[MAXV > 0 ? MAXV : 1];
    const int nvec = K / IV::N;

    // ---- pass 1: absmax (Alg. 1, dynamic quantisation scale)
    float amax = 0.0f;
    if constexpr (MAXV > 0) {
        const typename IV::V* xv = reinterpret_cast<const typename IV::V*>(x);
#pragma unroll
        for (int i = 0; i < MAXV; ++i) {
            const int idx = t + i * THREADS;
            if (idx < nvec) {
                v[i] = xv[idx];
                if constexpr (OUT < 2) {
                    float f[IV::N]; IV::unpack(v[i], f);
#pragma unroll
                    for (int e = 0; e < IV::N; ++e) amax = fmaxf(amax, fabsf(f[e]));
                }
            }
        }
    } else if constexpr (OUT < 2) {
        for (int k = t; k < K; k += THREADS) amax = fmaxf(amax, fabsf(load_scalar(x + k)));
    }
    float r = 0.0f;
    if constexpr (OUT < 2) {
        amax = block_absmax<THREADS>(amax, red);
        constexpr float QMAX = OUT == 0 ? 127.0f : 448.0f;
        float s = 1.0f;
        if (amax > 0.0f) { r = QMAX / amax; s = amax / QMAX; }
        if (t == 0) s_x[m] = s;
    }

    // ---- N = 2 from registers: plain quantisation has no windows to gather, so the quantised vectors go straight to
    // global memory (4 or 8 bytes per lane, contiguous across the wavefront) without the round trip through LDS
    if constexpr (MAXV > 0) {
        if (N == 2) {
            constexpr int OW = IV::N * ES / 4;           // output dwords per input vector: 1 (fp32 -> 8 bit), 2, 2 or 4
            uint32_t* out32 = reinterpret_cast<uint32_t*>(XL + m * (int64_t)Kp * ES);
#pragma unroll
            for (int i = 0; i < MAXV; ++i) {
                const int idx = t + i * THREADS;
                if (idx < nvec) {
                    float f[IV::N]; IV::unpack(v[i], f);
                    uint32_t w[OW];
#pragma unroll
                    for (int k = 0; k < OW; ++k) {
                        if constexpr (ES == 1)
                            w[k] = quant1<OUT>(f[4 * k], r) | (quant1<OUT>(f[4 * k + 1], r) << 8) | (quant1<OUT>(f[4 * k + 2], r) << 16) |
                                   (quant1<OUT>(f[4 * k + 3], r) << 24);
                        else
                            w[k] = quant1<OUT>(f[2 * k], r) | (quant1<OUT>(f[2 * k + 1], r) << 16);
                    }
                    if constexpr (OW == 1) out32[idx] = w[0];
                    else if constexpr (OW == 2) reinterpret_cast<uint2*>(out32)[idx] = make_uint2(w[0], w[1]);
                    else reinterpret_cast<uint4*>(out32)[idx] = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
            // zero padding of the stored width (K is a whole number of vectors here, so of dwords too)
            for (int k = K * ES / 4 + t; k < Kp * ES / 4; k += THREADS) out32[k] = 0u;
            return;
        }
    }

    // ---- pass 2a: quantise every source element once, into LDS
    if constexpr (MAXV > 0) {
#pragma unroll
        for (int i = 0; i < MAXV; ++i) {
            const int idx = t + i * THREADS;
            if (idx < nvec) {
                float f[IV::N]; IV::unpack(v[i], f);
                if constexpr (ES == 1) {
#pragma unroll
                    for (int w = 0; w < IV::N / 4; ++w) {
                        uint32_t p = quant1<OUT>(f[4 * w], r) | (quant1<OUT>(f[4 * w + 1], r) << 8) |
                                     (quant1<OUT>(f[4 * w + 2], r) << 16) | (quant1<OUT>(f[4 * w + 3], r) << 24);
                        lds[idx * (IV::N / 4) + w] = p;
                    }
                } else {
#pragma unroll
                    for (int w = 0; w < IV::N / 2; ++w)
                        lds[idx * (IV::N / 2) + w] = quant1<OUT>(f[2 * w], r) | (quant1<OUT>(f[2 * w + 1], r) << 16);
                }
            }
        }
    } else {
        if constexpr (ES == 1) {
            uint8_t* l8 = reinterpret_cast<uint8_t*>(lds);
            for (int k = t; k < K; k += THREADS) l8[k] = (uint8_t)quant1<OUT>(load_scalar(x + k), r);
        } else {
            uint16_t* l16 = reinterpret_cast<uint16_t*>(lds);
            for (int k = t; k < K; k += THREADS) l16[k] = (uint16_t)quant1<OUT>(load_scalar(x + k), r);
        }
    }
    if constexpr (ES == 1) {
        uint8_t* l8 = reinterpret_cast<uint8_t*>(lds);
        for (int k = K + t; k < Kz; k += THREADS) l8[k] = 0;
    } else {
        uint16_t* l16 = reinterpret_cast<uint16_t*>(lds);
        for (int k = K + t; k < Kz; k += THREADS) l16[k] = 0;
    }
    __syncthreads();

    // ---- pass 2b: output-oriented gather of the lifted windows (window j reads b = 2N g + 2 l);
    // windows at and beyond n_w = n_g (N-1) are the zero padding of the last 128-byte unit
    const int nw1 = N - 1;
    const int nwin = Kp / 4;
    const int ng = (K + 2 * N - 1) / (2 * N);
    uint4* out = reinterpret_cast<uint4*>(XL + m * (int64_t)Kp * ES);
    if constexpr (ES == 1) {
        for (int c = t; c < nwin / 4; c += THREADS) {
            int j = 4 * c, g = j / nw1, l = j - g * nw1;
            uint32_t w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                w[i] = 0;
                if (g < ng) {
                    const int b = 2 * N * g + 2 * l;
                    const uint32_t lo = lds[b >> 2], hi = lds[(b >> 2) + 1];
                    w[i] = (b & 2) ? ((lo >> 16) | (hi << 16)) : lo;
                }
                if (++l == nw1) { l = 0; ++g; }
            }
            out[c] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    } else {
        // 16-bit elements: a window is 8 bytes = elements b..b+3, b even -> two aligned dwords
        for (int c = t; c < nwin / 2; c += THREADS) {
            int j = 2 * c, g = j / nw1, l = j - g * nw1;
            uint32_t w[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                w[2 * i] = 0; w[2 * i + 1] = 0;
                if (g < ng) {
                    const int b = 2 * N * g + 2 * l;
                    w[2 * i] = lds[b >> 1]; w[2 * i + 1] = lds[(b >> 1) + 1];
                }
                if (++l == nw1) { l = 0; ++g; }
            }
            out[c] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

// elements of the quantised row kept in LDS: whole blocks plus 8 bytes that the gather may read
// past the last window, rounded to whole dwords
static inline int64_t lift_lds_elems(int64_t K, int N, int es) { return (n_groups(K, N) * 2 * N * es + 8 + 3) / 4 * 4 / es; }

template <typename TIN, int OUT>
static ss_status launch_lift(const void* X, int64_t M, int64_t K, int64_t ldx, int N, void* XL, float* s_x, hipStream_t st)
{
    typedef InVec<TIN> IV;
    const int ES = OUT >= 2 ? 2 : 1;
    const int Kp = (int)lifted_ld(K, N, ES);
    const int Kz = (int)lift_lds_elems(K, N, ES);
    const size_t lds_bytes = (size_t)Kz * ES;
    const bool vec_ok = (K % IV::N == 0) && (ldx % IV::N == 0) && (((uintptr_t)X & 15) == 0);
    const int64_t nvec = K / IV::N;                           // 16-byte vectors per row
    dim3 grid((unsigned)M);
    const TIN* x = static_cast<const TIN*>(X);
    uint8_t* xl = static_cast<uint8_t*>(XL);
#define SS_LQ(MAXV, T) hipLaunchKernelGGL((k_act_lift_quant<TIN, OUT, MAXV, T>), grid, dim3(T), lds_bytes, st, x, ldx, (int)K, N, xl, s_x, Kp, Kz)
    if (vec_ok && nvec <= 4 * 256) SS_LQ(4, 256);
    else if (vec_ok && nvec <= 4 * 512) SS_LQ(4, 512);
    else if (vec_ok && nvec <= 5 * 1024) SS_LQ(5, 1024);
    else if (vec_ok && nvec <= 10 * 1024) SS_LQ(10, 1024);
    else if (vec_ok && nvec <= 20 * 1024) SS_LQ(20, 1024);
    else SS_LQ(0, 256);
#undef SS_LQ
    return launch_status();
}

// ------------------------------------------------------------------------------------------
// Offline: magnitude pruning to (2N-2):2N followed by per-output-channel quantisation.
// One workgroup per weight row; thread per 2N block in the second pass.
template <typename TIN, int OUT>
__global__ __launch_bounds__(LQ_THREADS) void k_prune_quant(const TIN* __restrict__ W, int K, int N, uint8_t* __restrict__ Wq,
                                                             float* __restrict__ s_w)
{
    constexpr int ES = OUT >= 2 ? 2 : 1;
    __shared__ float red[LQ_THREADS / 64];
    const int64_t o = blockIdx.x;
    const TIN* w = W + o * (int64_t)K;
    const int t = threadIdx.x;
    float r = 0.0f;
    if constexpr (OUT < 2) {
        float amax = 0.0f;
        for (int k = t; k < K; k += LQ_THREADS) amax = fmaxf(amax, fabsf(load_scalar(w + k)));
        amax = block_absmax<LQ_THREADS>(amax, red);   // the row maximum always survives pruning
        constexpr float QMAX = OUT == 0 ? 127.0f : 448.0f;
        float s = 1.0f;
        if (amax > 0.0f) { r = QMAX / amax; s = amax / QMAX; }
        if (t == 0) s_w[o] = s;
    }
    const int L = 2 * N, ng = (K + L - 1) / L;            // a partial last block is completed with zeros
    for (int g = t; g < ng; g += LQ_THREADS) {
        float v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = (k < L && g * L + k < K) ? load_scalar(w + g * L + k) : 0.0f;
        // the two entries dropped are the last two in the order (|w| descending, index ascending)
        int d1 = 0, d2 = -1;
        float m1 = fabsf(v[0]);
#pragma unroll
        for (int k = 1; k < 16; ++k) if (k < L && fabsf(v[k]) <= m1) { m1 = fabsf(v[k]); d1 = k; }
        float m2 = 0.0f;
#pragma unroll
        for (int k = 0; k < 16; ++k) if (k < L && k != d1 && (d2 < 0 || fabsf(v[k]) <= m2)) { m2 = fabsf(v[k]); d2 = k; }
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            if (k < L && g * L + k < K) {
                const uint32_t q = (k == d1 || k == d2) ? 0u : quant1<OUT>(v[k], r);
                if constexpr (ES == 1) Wq[o * (int64_t)K + g * L + k] = (uint8_t)q;
                else reinterpret_cast<uint16_t*>(Wq)[o * (int64_t)K + g * L + k] = (uint16_t)q;
            }
        }
    }
}

}  // namespace ss

using namespace ss;

extern "C" int64_t slide_lifted_k(int64_t K, int N)
{
    if (!valid_N(N) || K <= 0 || K > (1 << 24)) return -1;
    return lifted_k(K, N);
}

extern "C" int64_t slide_lifted_ld(int64_t K, int N, ss_dtype dtype)
{
    if (!valid_N(N) || K <= 0 || K > (1 << 24) || !valid_dtype(dtype)) return -1;
    return lifted_ld(K, N, elem_size(dtype));
}

extern "C" ss_status act_lift_quant(const void* X, ss_act_dtype in_dtype, int64_t M, int64_t K, int64_t ldx, int N,
                                    ss_dtype out, void* X_lifted, float* s_x, void* stream)
{
    if (!valid_N(N)) return SS_ERR_BAD_PATTERN_N;
    if (M < 0 || K <= 0 || ldx < K || K > (1 << 24) || M > 0x7FFFFFFF) return SS_ERR_SHAPE;
    if (in_dtype != SS_IN_F32 && in_dtype != SS_IN_BF16) return SS_ERR_DTYPE;
    if (!valid_dtype(out)) return SS_ERR_DTYPE;
    // the quantised row and the kernel's small reduction buffer (at most 64 bytes) must fit in 64 KiB of LDS
    if ((size_t)lift_lds_elems(K, N, elem_size(out)) * elem_size(out) + 64 > 64 * 1024) return SS_ERR_SHAPE;
    if (M == 0) return SS_OK;
    if (!X || !X_lifted || (!unscaled(out) && !s_x)) return SS_ERR_NULL;
    if ((uintptr_t)X_lifted & 15) return SS_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (in_dtype == SS_IN_F32) {
        if (out == SS_I8) return launch_lift<float, 0>(X, M, K, ldx, N, X_lifted, s_x, st);
        if (out == SS_FP8_E4M3) return launch_lift<float, 1>(X, M, K, ldx, N, X_lifted, s_x, st);
        if (out == SS_BF16) return launch_lift<float, 2>(X, M, K, ldx, N, X_lifted, s_x, st);
        return launch_lift<float, 3>(X, M, K, ldx, N, X_lifted, s_x, st);
    }
    if (out == SS_I8) return launch_lift<uint16_t, 0>(X, M, K, ldx, N, X_lifted, s_x, st);
    if (out == SS_FP8_E4M3) return launch_lift<uint16_t, 1>(X, M, K, ldx, N, X_lifted, s_x, st);
    if (out == SS_BF16) return launch_lift<uint16_t, 2>(X, M, K, ldx, N, X_lifted, s_x, st);
    return launch_lift<uint16_t, 3>(X, M, K, ldx, N, X_lifted, s_x, st);
}

template <typename TIN, int OUT>
static ss_status launch_prune(const void* W, int64_t O, int64_t K, int N, void* Wq, float* s_w, hipStream_t st)
{
    hipLaunchKernelGGL((k_prune_quant<TIN, OUT>), dim3((unsigned)O), dim3(LQ_THREADS), 0, st, static_cast<const TIN*>(W), (int)K, N,
                       static_cast<uint8_t*>(Wq), s_w);
    return launch_status();
}

extern "C" ss_status slide_prune_quant(const void* W, ss_act_dtype in_dtype, int64_t O, int64_t K, int N, ss_dtype dtype,
                                       void* Wq, float* s_w, void* stream)
{
    if (!valid_N(N)) return SS_ERR_BAD_PATTERN_N;
    if (O < 0 || K <= 0 || K > (1 << 24) || O > 0x7FFFFFFF) return SS_ERR_SHAPE;
    if (in_dtype != SS_IN_F32 && in_dtype != SS_IN_BF16) return SS_ERR_DTYPE;
    if (!valid_dtype(dtype)) return SS_ERR_DTYPE;
    if (O == 0) return SS_OK;
    if (!W || !Wq || (!unscaled(dtype) && !s_w)) return SS_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (in_dtype == SS_IN_F32) {
        if (dtype == SS_I8) return launch_prune<float, 0>(W, O, K, N, Wq, s_w, st);
        if (dtype == SS_FP8_E4M3) return launch_prune<float, 1>(W, O, K, N, Wq, s_w, st);
        if (dtype == SS_BF16) return launch_prune<float, 2>(W, O, K, N, Wq, s_w, st);
        return launch_prune<float, 3>(W, O, K, N, Wq, s_w, st);
    }
    if (dtype == SS_I8) return launch_prune<uint16_t, 0>(W, O, K, N, Wq, s_w, st);
    if (dtype == SS_FP8_E4M3) return launch_prune<uint16_t, 1>(W, O, K, N, Wq, s_w, st);
    if (dtype == SS_BF16) return launch_prune<uint16_t, 2>(W, O, K, N, Wq, s_w, st);
    return launch_prune<uint16_t, 3>(W, O, K, N, Wq, s_w, st);
}
