// Matrix instructions of gfx950 per operand type, shared by the GEMM kernels.
#pragma once
#include "ss_common.h"

namespace ss {

// Sparse: one instruction is 32 channels x 32 tokens x 64 lifted bytes (A = 16 bytes of stored values + an
// index word per lane, B = 32 bytes per lane).  Dense: DENSE_SUB k-bytes per instruction, A and B
// DENSE_SUB / 2 bytes per lane; lane (row, q) holds the bytes [q DENSE_SUB / 2, (q + 1) DENSE_SUB / 2) of
// its row within the instruction's k range, for both operands (measured: element e of A lane (i, q)
// meets element e of B lane (n, q)).
template <int DT> struct Mma;
template <> struct Mma<SS_I8> {
    typedef v16i acc_t;
    typedef v4i dfrag_t;
    static constexpr int DENSE_SUB = 32;
    static constexpr bool SCALED = true;
    __device__ static acc_t sparse(v4i a, v8i b, acc_t c, int idx) { return __builtin_amdgcn_smfmac_i32_32x32x64_i8(a, b, c, idx, 0, 0); }
    __device__ static acc_t dense(dfrag_t a, dfrag_t b, acc_t c) { return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }
};
template <> struct Mma<SS_FP8_E4M3> {
    typedef v16f acc_t;
    typedef v8i dfrag_t;
    static constexpr int DENSE_SUB = 64;
    static constexpr bool SCALED = true;
    __device__ static acc_t sparse(v4i a, v8i b, acc_t c, int idx) { return __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(a, b, c, idx, 0, 0); }
    // format selectors 0 = e4m3 for both operands; block scales 0 = the unscaled form of the instruction
    __device__ static acc_t dense(dfrag_t a, dfrag_t b, acc_t c) { return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0); }
};
template <> struct Mma<SS_BF16> {
    typedef v16f acc_t;
    typedef v4i dfrag_t;
    static constexpr int DENSE_SUB = 32;
    static constexpr bool SCALED = false;
    __device__ static acc_t sparse(v4i a, v8i b, acc_t c, int idx)
    {
        return __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v16bf, b), c, idx, 0, 0);
    }
    __device__ static acc_t dense(dfrag_t a, dfrag_t b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
    }
};

template <> struct Mma<SS_FP16> {
    typedef v16f acc_t;
    typedef v4i dfrag_t;
    static constexpr int DENSE_SUB = 32;
    static constexpr bool SCALED = false;
    // same operand geometry as bf16 (checked by the parity tests against the oracle)
    __device__ static acc_t sparse(v4i a, v8i b, acc_t c, int idx)
    {
        return __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v16h, b), c, idx, 0, 0);
    }
    __device__ static acc_t dense(dfrag_t a, dfrag_t b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
    }
};

// two fp32 -> packed bf16 (round to nearest even) in one v_cvt_pk_bf16_f32
__device__ inline uint32_t pack_bf16x2(float a, float b)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Kernels for few tokens (gemm_skinny.hip).  The C entry points choose them for M <= 64, and for M <= 128 when
// the 256 x 256 tile kernels would have fewer than 64 tiles to spread over the compute units (measured on the
// Qwen2.5-7B shapes at M = 128: 26 vs 32 us for 3584 -> 4608, but 84 vs 38 us for 3584 -> 37888).
constexpr int64_t SS_SKINNY_MAX_M = 128;
inline bool use_skinny(int64_t M, int64_t O) { return M <= 64 || (M <= SS_SKINNY_MAX_M && (O + 255) / 256 < 64); }
ss_status launch_sparse_skinny(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                               int64_t Kpb, ss_dtype dtype, void* Y, int64_t ldy, hipStream_t stream);
ss_status launch_dense_skinny(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, ss_dtype dtype,
                              void* Y, int64_t ldy, hipStream_t stream);

}  // namespace ss
