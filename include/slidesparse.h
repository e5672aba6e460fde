/*
 * slidesparse.h -- C ABI of the MI355X (gfx950) SlideSparse linear-layer library.
 *
 * The library computes the (2N-2):2N structured-sparse linear layer
 *        Y[M,O] = X[M,K] . W[O,K]^T
 * using only 2:4-sparse matrix instructions, following the paper's problem statement
 * (Sec. 3.1, goal equation  w^T x = Phi(w)^T Psi(x)):
 *   Phi  = Sliding Window Decomposition of the weights   (Sec. 3.2, Alg. 2)  -> slide_decompose
 *   Psi  = Activation Lifting fused into per-token quantisation (Sec. 3.3, Alg. 1) -> act_lift_quant
 *   2:4 sparse GEMM over the lifted width K' = K*2(N-1)/N (Sec. 4.3)        -> slide_sparse_gemm
 *   dense GEMM at the original K, the baseline of every speed-up (Sec. 5.1)  -> dense_gemm
 *
 * Symbols: M tokens, K input features, O output features, N pattern parameter of
 * the (2N-2):2N pattern (N = 2 is native 2:4), K' the lifted width, Kld >= K' the stored
 * width of a lifted row (slide_lifted_ld).  K need not be a multiple of 2N: as in Alg. 1
 * (n_g = ceil(K/2N)) the last block is completed with zeros.
 *
 * Conventions for every call
 *   - every data pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates, frees or keeps a pointer after the call returns (scratch memory, where a
 *     call can use it, is passed in by the caller);
 *   - work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default
 *     stream) and the call returns without synchronising;
 *   - arguments are validated on the host before anything is enqueued; a bad argument
 *     returns an error code and enqueues nothing; there are no exceptions or aborts;
 *   - outputs are overwritten completely; inputs are read-only and must not alias
 *     outputs;
 *   - all matrices are row-major and dense unless a leading dimension is given.
 */
#ifndef SLIDESPARSE_H
#define SLIDESPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SS_OK = 0,
    SS_ERR_NULL = 1,           /* a required pointer is NULL                                  */
    SS_ERR_BAD_PATTERN_N = 2,  /* N outside 2..8                                              */
    SS_ERR_SHAPE = 3,          /* a size is non-positive or violates a divisibility rule      */
    SS_ERR_DTYPE = 4,          /* unknown or unsupported dtype for this call                  */
    SS_ERR_WORKSPACE = 5,      /* workspace pointer not 16-byte aligned                       */
    SS_ERR_HIP = 6,            /* the HIP runtime reported an error at launch                 */
    SS_ERR_SCRATCH = 7         /* slide_sparse_gemm_static: the shape needs more scratch than the static buffer holds */
} ss_status;

/* operand storage type of the GEMM inputs */
typedef enum {
    SS_I8 = 0,        /* int8, symmetric, Qmax = 127, int32 accumulation                      */
    SS_FP8_E4M3 = 1,  /* OCP e4m3fn byte, Qmax = 448, fp32 accumulation                       */
    SS_BF16 = 2,      /* bfloat16, unscaled, fp32 accumulation                                */
    SS_FP16 = 3       /* IEEE half, unscaled, fp32 accumulation (finite values within +-65504) */
} ss_dtype;

/* storage type of the un-quantised activations / weights handed to the quantisers */
typedef enum { SS_IN_F32 = 0, SS_IN_BF16 = 1 } ss_act_dtype;

/* K' = 4 n_w = ceil(K/2N) * 4(N-1), the lifted width (Alg. 1; = K * 2(N-1)/N when 2N divides
 * K: Sec. 3.4, expansion factor gamma = 2 - 2/N).  Returns -1 if N is outside 2..8 or K is
 * outside 1..2^24. */
int64_t slide_lifted_k(int64_t K, int N);

/* Kld (Alg. 1: a lifted row is n_w packed windows = 4 n_w elements; the library stores it padded): the width, in
 * elements, of the rows act_lift_quant writes and of the K_lifted argument
 * of slide_sparse_gemm: K' rounded up to a whole number of 128-byte units (the k granularity
 * of the GEMM kernels).  Columns K' .. Kld-1 of X_lifted are zero and the matching windows of
 * the packed weights are empty, so they add nothing to the product.  Kld == K' for every
 * benchmark shape of the paper's models at 6:8.  Returns -1 on a bad N, K or dtype. */
int64_t slide_lifted_ld(int64_t K, int N, ss_dtype dtype);

/* Byte sizes of the two buffers slide_decompose writes for an [O,K] weight matrix (Sec. 4.3: the compressed
 * form holds only the non-zeros plus compact index metadata; Sec. 3.4 for the (N-1)/N count).
 * The packed layout is opaque (ordered for the sparse matrix instruction's operand and
 * index registers); rows are padded to a multiple of 128.  With b = bytes per element,
 * vals_bytes = Opad * Kld * b / 2 ((N-1)/N of the dense weight bytes when Kld = K') and
 * meta_bytes = Opad * Kld * b / 8 (one 4-byte index word per 16 bytes of values). */
ss_status slide_packed_sizes(int64_t O, int64_t K, int N, ss_dtype dtype,
                             size_t* vals_bytes, size_t* meta_bytes);

/* Offline weight preparation (Sec. 4.1 "prune", App. E magnitude pruning; per-output-
 * channel symmetric quantisation as in Alg. 1 pass 1): for every row o of W[O,K] keep the
 * 2N-2 largest-|w| entries of each aligned run of 2N (ties keep the lower index), then
 * s_w[o] = max|w|/Qmax and Wq = clamp(rne(w * (Qmax/max|w|))) (BF16: rne to bf16, s_w
 * untouched and may be NULL; FP16 likewise with rne to half).  W is fp32 or bf16
 * (in_dtype).  An all-zero row gets s_w = 1.  A last run shorter than 2N is treated as
 * completed with zeros, which are the first entries to be dropped. */
ss_status slide_prune_quant(const void* W, ss_act_dtype in_dtype, int64_t O, int64_t K, int N,
                            ss_dtype dtype, void* Wq, float* s_w, void* stream);

/* Sliding Window Decomposition + 2:4 compression (Sec. 3.2, Alg. 2; Sec. 4.3).
 * Wq[O,K] holds quantised weights obeying the (2N-2):2N pattern (at most 2N-2 non-zeros
 * per aligned run of 2N along K; +-0 count as zero for fp8/bf16/fp16).  Each 2N block is
 * rewritten as N-1 stride-2 windows of 4 by the greedy residual allocation (window order
 * g, l ascending; inside a window the first <=2 unused non-zeros in ascending position),
 * every window is stored as 2 values + two 2-bit positions, and the result is laid out
 * for slide_sparse_gemm (Kld wide; a last block shorter than 2N is completed with zeros).
 * violations (nullable, device int32, must be zeroed by the caller): incremented once
 * per 2N block that holds more than 2N-2 non-zeros; output is unspecified for such blocks. */
ss_status slide_decompose(const void* Wq, int64_t O, int64_t K, int N, ss_dtype dtype,
                          void* w_vals, void* w_meta, int32_t* violations, void* stream);

/* Same decomposition in a plain, documented form for inspection and parity tests:
 * vals[O, K'/2] (dtype) and idx[O, K'/4] bytes (K', not Kld), one per window = i0 | i1 << 2 with
 * i0 < i1 the positions (0..3) of the two stored values; a window with fewer than two
 * non-zeros stores value 0 at the lowest positions not holding a non-zero. */
ss_status slide_decompose_canonical(const void* Wq, int64_t O, int64_t K, int N, ss_dtype dtype,
                                    void* vals, uint8_t* idx, int32_t* violations, void* stream);

/* Fused quantisation + slide (Alg. 1).  X[M,K] with row stride ldx (elements), fp32 or
 * bf16.  Per token i: a = max_k |x|, s_x[i] = a/Qmax, r = Qmax/a (fp32), and for every
 * output window j = g(N-1)+l the four elements at b = 2N g + 2l are quantised as
 * clamp(rne(x*r), +-Qmax) and stored at X_lifted[i, 4j .. 4j+3].  out = SS_BF16 / SS_FP16: no
 * scaling, elements are rounded (rne) to bf16 / half and s_x may be NULL.  N = 2 is plain
 * per-token quantisation (K' = K rounded up to 4).  An all-zero token gets s_x = 1 and
 * zeros.  Source columns at or beyond K read as zero.  X_lifted is [M, Kld] dense, 16-byte
 * aligned (SS_ERR_SHAPE otherwise), columns K'..Kld-1 zero.  The quantised row is kept in
 * on-chip memory: ceil(K/2N)*2N*sizeof(element) + 72 must not exceed 64 KiB (SS_ERR_SHAPE otherwise). */
ss_status act_lift_quant(const void* X, ss_act_dtype in_dtype, int64_t M, int64_t K, int64_t ldx,
                         int N, ss_dtype out, void* X_lifted, float* s_x, void* stream);

/* 2:4 sparse GEMM over the lifted width (Sec. 4.3) with the scale epilogue:
 *   Y[m,o] = bf16( (fp32(acc[m,o]) * s_x[m]) * s_w[o] ),  acc = sum over K' of X' . W'
 * (SS_BF16, SS_FP16: Y = bf16(acc), s_x and s_w ignored and may be NULL).  X_lifted[M,K_lifted]
 * dense row-major from act_lift_quant (K_lifted = Kld); w_vals/w_meta from slide_decompose
 * for the same O, K and N.  Y is bf16 [M,O] with row stride ldy (elements, O <= ldy < 2^22).  INT8 accumulates
 * in int32 (exact), FP8, BF16 and FP16 in fp32 in the order of the matrix instructions (the fp8
 * instructions of gfx950 add the products of one instruction in groups aligned to the group's
 * largest product, keeping 14 bits below it; bf16 / fp16 products keep all 24).
 * Requires K_lifted * sizeof(element) % 128 == 0 (and <= 2^23 bytes per row), M <= 2^24, and 16-byte
 * aligned operand pointers.  Three kernel families are chosen from M, O and K_lifted: kernels that
 * stream the weights once (few tokens), 128 x 128 tiles (shapes too small to fill the chip with
 * large tiles) and persistent 256 x 256 tiles; results are the same (INT8) or differ in fp32
 * summation order only.  Every call with the same arguments gives the same bits. */
ss_status slide_sparse_gemm(const void* X_lifted, const float* s_x, const void* w_vals,
                            const void* w_meta, const float* s_w, int64_t M, int64_t O,
                            int64_t K_lifted, ss_dtype dtype, void* Y, int64_t ldy, void* stream);

/* Dense baseline at the original K with the same epilogue: Xq[M,K], Wq[O,K] row-major.
 * Requires K * sizeof(element) % 128 == 0 (and <= 2^23 bytes per row), M <= 2^24, O <= ldy < 2^22, and
 * 16-byte aligned operand pointers. */
ss_status dense_gemm(const void* Xq, const float* s_x, const void* Wq, const float* s_w,
                     int64_t M, int64_t O, int64_t K, ss_dtype dtype, void* Y, int64_t ldy,
                     void* stream);

/* The same two GEMMs with a caller-owned scratch buffer (Sec. 5 measures from decode, M = 64, to
 * prefill; small M leaves most of the chip idle unless the k range is split).  With a workspace of
 * at least slide_gemm_workspace_bytes() the 128 x 128-tile kernels (and the few-token kernels on
 * long rows) split the k range of a tile over several workgroups, write fp32 / int32 partial
 * sums to the workspace and add them in a fixed order in a second kernel (bit-reproducible; INT8 results are identical to the calls
 * without workspace).  workspace: device memory, 16-byte aligned (SS_ERR_WORKSPACE otherwise),
 * contents irrelevant before and undefined after; NULL with workspace_bytes = 0, or a smaller
 * buffer, is allowed and gives fewer or no splits.  Calls that share one workspace must be ordered
 * on one stream.  K is the row length in elements as passed to the GEMM (K_lifted for the sparse
 * one); the function returns 0 when the shape would not be split or an argument is invalid. */
size_t slide_gemm_workspace_bytes(int64_t M, int64_t O, int64_t K, ss_dtype dtype);
ss_status slide_sparse_gemm_ws(const void* X_lifted, const float* s_x, const void* w_vals,
                               const void* w_meta, const float* s_w, int64_t M, int64_t O,
                               int64_t K_lifted, ss_dtype dtype, void* Y, int64_t ldy,
                               void* workspace, size_t workspace_bytes, void* stream);
ss_status dense_gemm_ws(const void* Xq, const float* s_x, const void* Wq, const float* s_w,
                        int64_t M, int64_t O, int64_t K, ss_dtype dtype, void* Y, int64_t ldy,
                        void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): slide_sparse_gemm_ws with the scratch buffer in a static device array of
 * slide_static_scratch_bytes() = 16 MiB inside the library (every GPU the library runs on holds its own copy until the
 * process ends).  The call allocates and frees nothing.  Same arguments, kernels and results as slide_sparse_gemm_ws
 * given a workspace of slide_gemm_workspace_bytes(); a shape that would need more than the static buffer returns
 * SS_ERR_SCRATCH and enqueues nothing (16 MiB covers every shape on a device of up to 256 compute units).  All calls on
 * one GPU share that GPU's array: it holds the previous call's partial sums, every call overwrites the part it reads
 * (nothing needs clearing), and calls that overlap in time on one GPU (different streams) race on it; order them. */
size_t slide_static_scratch_bytes(void);
ss_status slide_sparse_gemm_static(const void* X_lifted, const float* s_x, const void* w_vals,
                                   const void* w_meta, const float* s_w, int64_t M, int64_t O,
                                   int64_t K_lifted, ss_dtype dtype, void* Y, int64_t ldy, void* stream);

/* Fused lifting (Sec. 3.3 lifting operator realised inside the GEMM; the paper fuses it into quantisation, Alg. 1):
 * the same linear layer for the 6:8 pattern (N = 4; any other N returns SS_ERR_BAD_PATTERN_N) computed from the
 * UNLIFTED quantised activations Xq[M,K] (row stride ldx elements; what act_lift_quant writes with N = 2), so the
 * lifted matrix is never materialised.  The weights are packed by slide_decompose_fused, which runs the same
 * decomposition as slide_decompose (Alg. 2) but orders the windows for this kernel (opaque; sizes from
 * slide_packed_sizes_fused); buffers of the two packers are not interchangeable.  Requires K * sizeof(element) % 128 == 0
 * (pad X and W with zero columns otherwise), ldx * sizeof(element) % 16 == 0, 16-byte aligned pointers, O <= ldy < 2^22,
 * M <= 2^24.  Same epilogue, accumulation rules and error behaviour as slide_sparse_gemm; INT8 results are identical
 * to slide_sparse_gemm and dense_gemm, floating-point results differ in summation order only. */
ss_status slide_packed_sizes_fused(int64_t O, int64_t K, int N, ss_dtype dtype, size_t* vals_bytes, size_t* meta_bytes);
ss_status slide_decompose_fused(const void* Wq, int64_t O, int64_t K, int N, ss_dtype dtype,
                                void* w_vals, void* w_meta, int32_t* violations, void* stream);
ss_status slide_sparse_gemm_fused(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta,
                                  const float* s_w, int64_t M, int64_t O, int64_t K, int64_t ldx, int N,
                                  ss_dtype dtype, void* Y, int64_t ldy, void* stream);
/* The fused GEMM with a caller-owned scratch buffer, as slide_sparse_gemm_ws (Sec. 5's token counts from decode to
 * prefill): for few tokens and for shapes with few tiles the same kernel families as the other GEMMs are used, with
 * the k loop counted in units of 128 unlifted bytes, and a workspace of slide_gemm_workspace_bytes(M, O, K, dtype)
 * bytes (K the unlifted row length, as for dense_gemm_ws) lets them split the k range.  workspace rules and error
 * behaviour as for slide_sparse_gemm_ws; slide_sparse_gemm_fused is this call without workspace. */
ss_status slide_sparse_gemm_fused_ws(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta,
                                     const float* s_w, int64_t M, int64_t O, int64_t K, int64_t ldx, int N,
                                     ss_dtype dtype, void* Y, int64_t ldy, void* workspace, size_t workspace_bytes,
                                     void* stream);

/* Library housekeeping (no passage of the paper): a static, human-readable name for a status code ... */
const char* ss_status_string(ss_status s);

/* ... and the version of the opaque packed layouts (Sec. 4.3 leaves the compressed format to the implementation;
 * bumped whenever what slide_decompose / slide_decompose_fused write changes). */
int slide_format_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SLIDESPARSE_H */
