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
    static constexpr int ES = 1;                       // bytes per element
    static constexpr int DENSE_SUB = 32;
    static constexpr bool SCALED = true;
    __device__ static acc_t sparse(v4i a, v8i b, acc_t c, int idx) { return __builtin_amdgcn_smfmac_i32_32x32x64_i8(a, b, c, idx, 0, 0); }
    __device__ static acc_t dense(dfrag_t a, dfrag_t b, acc_t c) { return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }
};
template <> struct Mma<SS_FP8_E4M3> {
    typedef v16f acc_t;
    typedef v8i dfrag_t;
    static constexpr int ES = 1;
    static constexpr int DENSE_SUB = 64;
    static constexpr bool SCALED = true;
    __device__ static acc_t sparse(v4i a, v8i b, acc_t c, int idx) { return __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(a, b, c, idx, 0, 0); }
    // format selectors 0 = e4m3 for both operands; block scales 0 = the unscaled form of the instruction
    __device__ static acc_t dense(dfrag_t a, dfrag_t b, acc_t c) { return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0); }
};
template <> struct Mma<SS_BF16> {
    typedef v16f acc_t;
    typedef v4i dfrag_t;
    static constexpr int ES = 2;
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
    static constexpr int ES = 2;
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

// Epilogue of one accumulator block held by one lane: a[r] is channel o_lane + r (16 consecutive channels) of token
// tok; Y = bf16((float(a) * s_x[tok]) * s_w[o]) (SCALED) or bf16(a).  Out-of-range tokens and channels are skipped.
template <bool SCALED, typename ACC>
__device__ inline void store_block16(const ACC& a, const float* __restrict__ s_x, const float* __restrict__ s_w, uint16_t* __restrict__ Y,
                                     int64_t ldy, int64_t M, int64_t O, int64_t o_lane, int64_t tok)
{
    if (tok >= M || o_lane >= O) return;
    uint32_t w[8];
    if constexpr (SCALED) {
        const float sx = s_x[tok];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int64_t o0 = o_lane + 2 * q, o1 = o0 + 1;
            w[q] = pack_bf16x2(((float)a[2 * q] * sx) * s_w[o0 < O ? o0 : O - 1], ((float)a[2 * q + 1] * sx) * s_w[o1 < O ? o1 : O - 1]);
        }
    } else {
#pragma unroll
        for (int q = 0; q < 8; ++q) w[q] = pack_bf16x2((float)a[2 * q], (float)a[2 * q + 1]);
    }
    uint16_t* dst = Y + tok * ldy + o_lane;
    if (((ldy & 7) == 0) && (((uintptr_t)Y & 15) == 0) && o_lane + 16 <= O) {
        reinterpret_cast<uint4*>(dst)[0] = make_uint4(w[0], w[1], w[2], w[3]);
        reinterpret_cast<uint4*>(dst)[1] = make_uint4(w[4], w[5], w[6], w[7]);
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (o_lane + e < O) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
    }
}

// Epilogue of four consecutive channels o .. o + 3 of token tok held by one thread (the split-k reduce kernels):
// Y = bf16((float(a) * s_x[tok]) * s_w[o]) (SCALED) or bf16(a).  Out-of-range tokens and channels are skipped.
template <bool SCALED, typename QUAD>
__device__ inline void store_quad4(const QUAD& a, const float* __restrict__ s_x, const float* __restrict__ s_w, uint16_t* __restrict__ Y,
                                   int64_t ldy, int64_t M, int64_t O, int64_t o, int64_t tok)
{
    if (tok >= M || o >= O) return;
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[e] = (float)a[e];
        if constexpr (SCALED) v[e] = (v[e] * s_x[tok]) * s_w[o + e < O ? o + e : O - 1];
    }
    const uint32_t w[2] = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
    uint16_t* dst = Y + tok * ldy + o;
    if (o + 4 <= O && (((uintptr_t)dst) & 7) == 0) *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
    else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (o + e < O) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
    }
}

// Kernels for few tokens (gemm_skinny.hip): one workgroup per 32..128 output channels streams their weights once.
// With S > 1 (only where every workgroup is a single 32-channel fragment and there are fewer of them than compute
// units) the k range is split over S workgroups per fragment; partial sums go through `ws`
// (skinny_workspace_bytes(M, O, S) bytes) and a second kernel adds them in a fixed order.
constexpr int64_t SS_SKINNY_MAX_M = 64;
int skinny_splits(int64_t M, int64_t O, int64_t units, size_t ws_bytes);
size_t skinny_workspace_bytes(int64_t M, int64_t O, int S);
ss_status launch_sparse_skinny(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                               int64_t Kpb, ss_dtype dtype, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream);
// the same for unlifted activations and weights packed by slide_decompose_fused (6:8): U super-units of 128 bytes per row,
// ldxb bytes between token rows
ss_status launch_sparse_fused_skinny(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                                     int U, int64_t ldxb, ss_dtype dtype, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream);
ss_status launch_dense_skinny(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, ss_dtype dtype,
                              void* Y, int64_t ldy, void* ws, int S, hipStream_t stream);


// The 256 x 256 tile kernels (gemm.hip).
ss_status launch_sparse_tile(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                             int64_t Kpb, ss_dtype dtype, void* Y, int64_t ldy, hipStream_t stream);
ss_status launch_dense_tile(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, ss_dtype dtype,
                            void* Y, int64_t ldy, hipStream_t stream);

// Kernels with 128 x 128 tiles (gemm_mid.hip) for shapes that give the 256 x 256 tile kernels too few tiles to
// occupy the compute units.
// S > 1 splits the k range over S workgroups per tile; their partial sums go through `ws`
// (mid_workspace_bytes(M, O, S) bytes) and a second kernel adds them in a fixed order.
ss_status launch_sparse_mid(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                            int64_t Kpb, ss_dtype dtype, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream);
// the same for unlifted activations and weights packed by slide_decompose_fused (6:8): U super-units of 128 bytes per row,
// ldxb bytes between token rows
ss_status launch_sparse_fused_mid(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                                  int U, int64_t ldxb, ss_dtype dtype, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream);
ss_status launch_dense_mid(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, ss_dtype dtype,
                           void* Y, int64_t ldy, void* ws, int S, hipStream_t stream);
int mid_splits(int64_t M, int64_t O, int64_t units, size_t ws_bytes);
size_t mid_workspace_bytes(int64_t M, int64_t O, int S);
inline int64_t mid_tiles(int64_t M, int64_t O) { return ((O + 127) / 128) * ((M + 127) / 128); }

// Which kernel family a GEMM of M tokens x O channels over `units` 128-byte k units runs on, and in how many k
// ranges (S > 1 only for SS_PATH_MID and only with a workspace).  Measured on the Qwen2.5-7B shapes (INT8, 6:8):
//   M <= 32                      few-token kernels (7 to 9 us on 3584 -> 4608, where the others need 15 and 31), their k
//                                range split in two or three where the fragments are fewer than the compute units and the
//                                rows long (18944 -> 3584);
//   32 < M <= 64                 the same, unless the rows are long and can be split (18944 -> 3584 at M = 48:
//                                53 us few-token, 23 us in 8 ranges of 128 x 128 tiles);
//   up to 320 tiles of 128 x 128 those tiles (M = 256 on 3584 -> 4608: 17 us in 3 ranges, 33 us with 256 x 256
//                                tiles; M = 1024 on 18944 -> 3584: 111 vs 150 us);
//   beyond                       the 256 x 256 tile kernels (M = 2048 on 3584 -> 4608: 40 vs 57 us).
enum ss_path { SS_PATH_SKINNY, SS_PATH_MID, SS_PATH_TILE };
struct ss_plan { ss_path path; int S; };
inline ss_plan plan_gemm(int64_t M, int64_t O, int64_t units, size_t ws_bytes)
{
    if (M <= 32) return {SS_PATH_SKINNY, skinny_splits(M, O, units, ws_bytes)};
    if (M > 64 && mid_tiles(M, O) > 320) return {SS_PATH_TILE, 1};
    const int S = mid_splits(M, O, units, ws_bytes);
    if (M <= 64 && !(S > 1 && units >= 96)) return {SS_PATH_SKINNY, skinny_splits(M, O, units, ws_bytes)};
    return {SS_PATH_MID, S};
}

}  // namespace ss
