// slide_sparse_gemm and dense_gemm for gfx950.
//
// Both kernels share one tile engine: a 512-thread workgroup (8 wavefronts, two per SIMD)
// owns a 256 (output channels) x 256 (tokens) tile of Y; wavefront (wo, wt) accumulates the
// 128 x 64 sub-tile [wo*128, +128) x [wt*64, +64) as 4 x 2 32x32 matrix-instruction blocks.
// Operand tiles stream HBM/L2 -> LDS with direct-to-LDS 16-byte loads through a ring of
// stages, so no registers are spent on data in flight; LDS rows are XOR-swizzled at 16-byte
// granularity (applied on the global-address side of the direct loads) so that the 32 lanes
// of a matrix-operand read hit all 64 banks.  The weights are the A operand (sparse for
// slide_sparse_gemm: v_smfmac_i32_32x32x64_i8 consumes 16 stored bytes + one index word per
// lane), tokens are the B operand, and the accumulator D[channel][token] leaves each lane
// with 64 consecutive output channels of one token, stored as full 128-byte lines.
#include "ss_common.h"
#include "packed_layout.h"

namespace ss {

constexpr int G_THREADS = 512;
constexpr int BO = 256;   // output channels per workgroup
constexpr int BT = 256;   // tokens per workgroup

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

__device__ inline void lds_dma16(const void* g, void* lds_wave_base)
{
    // 16 bytes per lane, global -> LDS; the LDS address is wave-uniform base + lane * 16
    __builtin_amdgcn_global_load_lds((gbl_void*)g, (lds_void*)lds_wave_base, 16, 0, 0);
}

template <int N> __device__ inline void wait_vmcnt()
{
    // gfx9 s_waitcnt encoding: vmcnt = bits [3:0] and [15:14]; leave expcnt / lgkmcnt at "no wait"
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// Workgroup barrier without the memory fence of __syncthreads(): the direct-to-LDS loads still in
// flight for later stages must stay in flight.  The empty asm statements keep the compiler from
// moving LDS reads or load issues across it.
__device__ inline void stage_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();     // stage kt has landed for every wave; stage kt-1 is no longer being read
    asm volatile("" ::: "memory");
}

// XCD-aware tile order: consecutive workgroup ids go round-robin to the 8 XCDs, so give each
// XCD one contiguous range of tiles, and order tiles in bands of 8 token tiles so the 32
// workgroups resident on an XCD share weight panels and token tiles in its L2.
__device__ inline void tile_of_block(int tiles_o, int tiles_t, int& to, int& tt)
{
    const int nb = gridDim.x, bid = blockIdx.x;
    const int xcd = bid & 7, idx = bid >> 3;
    const int q = nb >> 3, rem = nb & 7;
    const int tile = xcd * q + (xcd < rem ? xcd : rem) + idx;
    constexpr int BAND = 8;
    const int per_band = BAND * tiles_o;
    const int band = tile / per_band, within = tile - band * per_band;
    const int bw = min(BAND, tiles_t - band * BAND);
    to = within / bw;
    tt = band * BAND + (within - to * bw);
}

// ---- LDS tile of a row-major 8-bit operand: ROWS rows x KT bytes, XOR-swizzled -------------
template <int KT> __device__ inline int swz(int row) { return (row / (16 / (KT / 16))) % (KT / 16); }

// issue the direct-to-LDS loads of a [256 x KT] tile; rows >= nrows are clamped (their
// products are never stored)
template <int KT>
__device__ inline void load_rows_tile(const uint8_t* __restrict__ base, int64_t ld, int64_t row0, int64_t nrows, int64_t k0, uint8_t* lds_tile)
{
    constexpr int CPR = KT / 16;                 // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;                // rows per wavefront-wide load
    constexpr int NI = 256 / (RPI * (G_THREADS / 64));
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int r0 = (i * (G_THREADS / 64) + wave) * RPI;
        const int row = r0 + lane / CPR;
        const int lc = (lane % CPR) ^ swz<KT>(row);
        int64_t grow = row0 + row;
        grow = grow < nrows ? grow : nrows - 1;
        lds_dma16(base + grow * ld + k0 + lc * 16, lds_tile + r0 * KT);
    }
}

template <int KT> __device__ inline const v4i* tile_chunk(const uint8_t* lds_tile, int row, int lc)
{
    return reinterpret_cast<const v4i*>(lds_tile + row * KT + ((lc ^ swz<KT>(row)) << 4));
}

// ---- epilogue: Y = bf16((float(acc) * s_x) * s_w), 64 consecutive channels per lane ---------
__device__ inline uint32_t pack_bf16x2(float a, float b) { return (uint32_t)f32_to_bf16_bits(a) | ((uint32_t)f32_to_bf16_bits(b) << 16); }

template <typename ACC>
__device__ inline void store_tile(const ACC (&acc)[4][2], const float* __restrict__ s_x, const float* __restrict__ s_w, uint16_t* __restrict__ Y,
                                  int64_t ldy, int64_t M, int64_t O, int64_t o_base, int64_t t_base)
{
    const int lane = threadIdx.x & 63, n = lane & 31, h = lane >> 5;
    const int64_t o0 = o_base + 64 * h;
    const bool fast = (o0 + 64 <= O) && ((ldy & 7) == 0) && (((uintptr_t)Y & 15) == 0);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int64_t tok = t_base + b * 32 + n;
        if (tok >= M) continue;
        const float sx = s_x[tok];
        uint16_t* yrow = Y + tok * ldy + o0;
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            if (fast) {
                const float4* sw4 = reinterpret_cast<const float4*>(s_w + o0 + 16 * f);
                uint32_t w[8];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 sw = sw4[q];
                    w[2 * q] = pack_bf16x2(((float)acc[f][b][4 * q] * sx) * sw.x, ((float)acc[f][b][4 * q + 1] * sx) * sw.y);
                    w[2 * q + 1] = pack_bf16x2(((float)acc[f][b][4 * q + 2] * sx) * sw.z, ((float)acc[f][b][4 * q + 3] * sx) * sw.w);
                }
                uint4* dst = reinterpret_cast<uint4*>(yrow + 16 * f);
                dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
                dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t o = o0 + 16 * f + r;
                    if (o < O) yrow[16 * f + r] = f32_to_bf16_bits(((float)acc[f][b][r] * sx) * s_w[o]);
                }
            }
        }
    }
}

// ---- dense INT8: Y = Xq . Wq^T ----------------------------------------------------------------
constexpr int D_KT = 64, D_STAGES = 4, D_STAGE_BYTES = (BO + BT) * D_KT;

__global__ __launch_bounds__(G_THREADS) void k_dense_i8(const uint8_t* __restrict__ Xq, const float* __restrict__ s_x, const uint8_t* __restrict__ Wq,
                                                        const float* __restrict__ s_w, int64_t M, int64_t O, int64_t K, uint16_t* __restrict__ Y,
                                                        int64_t ldy, int tiles_o, int tiles_t)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    int to, tt;
    tile_of_block(tiles_o, tiles_t, to, tt);
    const int64_t o_blk = (int64_t)to * BO, t_blk = (int64_t)tt * BT;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wo = wave & 1, wt = wave >> 1;
    const int row = lane & 31, q = lane >> 5;
    const int nk = (int)(K / D_KT);
    constexpr int LPS = 2 * (256 / ((64 / (D_KT / 16)) * (G_THREADS / 64)));   // loads per thread per stage

    v16i acc[4][2];
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][b][r] = 0;

    auto issue = [&](int kt) {
        uint8_t* st = smem + (kt % D_STAGES) * D_STAGE_BYTES;
        load_rows_tile<D_KT>(Wq, K, o_blk, O, (int64_t)kt * D_KT, st);
        load_rows_tile<D_KT>(Xq, K, t_blk, M, (int64_t)kt * D_KT, st + BO * D_KT);
    };
#pragma unroll
    for (int s = 0; s < D_STAGES - 1; ++s) if (s < nk) issue(s);

    for (int kt = 0; kt < nk; ++kt) {
        if (kt + D_STAGES - 2 < nk) wait_vmcnt<(D_STAGES - 2) * LPS>(); else wait_vmcnt<0>();
        stage_barrier();
        if (kt + D_STAGES - 1 < nk) issue(kt + D_STAGES - 1);
        const uint8_t* sa = smem + (kt % D_STAGES) * D_STAGE_BYTES;
        const uint8_t* sb = sa + BO * D_KT;
#pragma unroll
        for (int u = 0; u < D_KT / 32; ++u) {
            v4i a[4], b[2];
#pragma unroll
            for (int f = 0; f < 4; ++f) a[f] = *tile_chunk<D_KT>(sa, wo * 128 + panel_row(f, row), 2 * u + q);
#pragma unroll
            for (int bb = 0; bb < 2; ++bb) b[bb] = *tile_chunk<D_KT>(sb, wt * 64 + bb * 32 + row, 2 * u + q);
#pragma unroll
            for (int f = 0; f < 4; ++f)
#pragma unroll
                for (int bb = 0; bb < 2; ++bb) acc[f][bb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[f], b[bb], acc[f][bb], 0, 0, 0);
        }
    }
    store_tile(acc, s_x, s_w, Y, ldy, M, O, o_blk + wo * 128, t_blk + wt * 64);
}

// ---- sparse INT8 over the lifted width: Y = X' . W'^T, W' packed 2:4 ----------------------------
constexpr int S_KT = 128, S_STAGES = 3;
constexpr int S_B_BYTES = BT * S_KT, S_AV_BYTES = BO * S_KT / 2, S_AM_BYTES = BO * S_KT / 8;
constexpr int S_STAGE_BYTES = S_B_BYTES + S_AV_BYTES + S_AM_BYTES;

__global__ __launch_bounds__(G_THREADS) void k_sparse_i8(const uint8_t* __restrict__ XL, const float* __restrict__ s_x, const uint8_t* __restrict__ w_vals,
                                                         const uint8_t* __restrict__ w_meta, const float* __restrict__ s_w, int64_t M, int64_t O,
                                                         int64_t Kp, uint16_t* __restrict__ Y, int64_t ldy, int tiles_o, int tiles_t)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    int to, tt;
    tile_of_block(tiles_o, tiles_t, to, tt);
    const int64_t o_blk = (int64_t)to * BO, t_blk = (int64_t)tt * BT;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wo = wave & 1, wt = wave >> 1;
    const int n = lane & 31, qb = lane >> 5;
    const int nk = (int)(Kp / S_KT);
    const int64_t nsteps = Kp / FRAG_K8;
    const int64_t npanels = (O + PANEL - 1) / PANEL;
    constexpr int LPS = 4 + 2 + 1;    // B: 4, A values: 2, A index words: 1 (issued by waves 0..3 only; they wait on one more)

    v16i acc[4][2];
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][b][r] = 0;

    auto issue = [&](int kt) {
        uint8_t* st = smem + (kt % S_STAGES) * S_STAGE_BYTES;
        load_rows_tile<S_KT>(XL, Kp, t_blk, M, (int64_t)kt * S_KT, st);
        // A values: per panel the two 64-column steps of this stage are 8 KB contiguous
#pragma unroll
        for (int pp = 0; pp < 2; ++pp) {
            int64_t panel = (int64_t)to * 2 + pp;
            panel = panel < npanels ? panel : npanels - 1;
            const uint8_t* src = w_vals + frag_slot(panel, nsteps, (int64_t)kt * 2, 0, 0) * 16;
            lds_dma16(src + threadIdx.x * 16, st + S_B_BYTES + pp * 8192 + wave * 1024);
        }
        // A index words: 2 KB contiguous per panel
        {
            const int w4 = wave & 3;
            int64_t panel = (int64_t)to * 2 + (w4 >> 1);
            panel = panel < npanels ? panel : npanels - 1;
            const uint8_t* src = w_meta + frag_slot(panel, nsteps, (int64_t)kt * 2, 0, 0) * 4 + (w4 & 1) * 1024;
            // waves 4..7 repeat the loads of waves 0..3 (same bytes, same LDS address) so that
            // every wave has the same number of loads in flight
            lds_dma16(src + lane * 16, st + S_B_BYTES + S_AV_BYTES + w4 * 1024);
        }
    };
#pragma unroll
    for (int s = 0; s < S_STAGES - 1; ++s) if (s < nk) issue(s);

    for (int kt = 0; kt < nk; ++kt) {
        if (kt + S_STAGES - 2 < nk) wait_vmcnt<(S_STAGES - 2) * LPS>(); else wait_vmcnt<0>();
        stage_barrier();
        if (kt + S_STAGES - 1 < nk) issue(kt + S_STAGES - 1);
        const uint8_t* sb = smem + (kt % S_STAGES) * S_STAGE_BYTES;
        const uint8_t* sav = sb + S_B_BYTES;
        const uint8_t* sam = sav + S_AV_BYTES;
#pragma unroll
        for (int u = 0; u < S_KT / 64; ++u) {
            v4i a[4]; int idx[4]; v8i b[2];
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const int fs = ((wo * 2 + u) * 4 + f) * 64 + lane;
                a[f] = *reinterpret_cast<const v4i*>(sav + fs * 16);
                idx[f] = *reinterpret_cast<const int*>(sam + fs * 4);
            }
#pragma unroll
            for (int bb = 0; bb < 2; ++bb) {
                const int r = wt * 64 + bb * 32 + n;
                const v4i lo = *tile_chunk<S_KT>(sb, r, 4 * u + 2 * qb);
                const v4i hi = *tile_chunk<S_KT>(sb, r, 4 * u + 2 * qb + 1);
                b[bb] = (v8i){lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
#pragma unroll
            for (int f = 0; f < 4; ++f)
#pragma unroll
                for (int bb = 0; bb < 2; ++bb) acc[f][bb] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(a[f], b[bb], acc[f][bb], idx[f], 0, 0);
        }
    }
    store_tile(acc, s_x, s_w, Y, ldy, M, O, o_blk + wo * 128, t_blk + wt * 64);
}

}  // namespace ss

using namespace ss;

static ss_status check_gemm(const void* X, const float* s_x, const void* W, const float* s_w, int64_t M, int64_t O, int64_t K,
                            ss_dtype dtype, const void* Y, int64_t ldy)
{
    if (dtype != SS_I8 && dtype != SS_FP8_E4M3 && dtype != SS_BF16) return SS_ERR_DTYPE;
    if (M < 0 || O < 0 || K <= 0 || K % KSTEP != 0 || ldy < O || M > (1 << 24) || O > (1 << 24) || K > (1 << 24)) return SS_ERR_SHAPE;
    if (dtype != SS_I8) return SS_ERR_DTYPE;          // fp8 / bf16 GEMMs not built yet
    if (M == 0 || O == 0) return SS_OK;
    if (!X || !W || !Y || !s_x || !s_w) return SS_ERR_NULL;
    if (((uintptr_t)X & 15) || ((uintptr_t)W & 15)) return SS_ERR_SHAPE;
    return SS_OK;
}

extern "C" ss_status dense_gemm(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t K,
                                ss_dtype dtype, void* Y, int64_t ldy, void* stream)
{
    ss_status st = check_gemm(Xq, s_x, Wq, s_w, M, O, K, dtype, Y, ldy);
    if (st != SS_OK || M == 0 || O == 0) return st;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)k_dense_i8, hipFuncAttributeMaxDynamicSharedMemorySize, D_STAGES * D_STAGE_BYTES) != hipSuccess) return SS_ERR_HIP;
        attr_set = true;
    }
    const int tiles_o = (int)((O + BO - 1) / BO), tiles_t = (int)((M + BT - 1) / BT);
    hipLaunchKernelGGL(k_dense_i8, dim3(tiles_o * tiles_t), dim3(G_THREADS), D_STAGES * D_STAGE_BYTES, static_cast<hipStream_t>(stream),
                       static_cast<const uint8_t*>(Xq), s_x, static_cast<const uint8_t*>(Wq), s_w, M, O, K, static_cast<uint16_t*>(Y), ldy,
                       tiles_o, tiles_t);
    return launch_status();
}

extern "C" ss_status slide_sparse_gemm(const void* X_lifted, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w,
                                       int64_t M, int64_t O, int64_t K_lifted, ss_dtype dtype, void* Y, int64_t ldy, void* stream)
{
    ss_status st = check_gemm(X_lifted, s_x, w_vals, s_w, M, O, K_lifted, dtype, Y, ldy);
    if (st != SS_OK || M == 0 || O == 0) return st;
    if (!w_meta) return SS_ERR_NULL;
    if ((uintptr_t)w_meta & 15) return SS_ERR_SHAPE;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)k_sparse_i8, hipFuncAttributeMaxDynamicSharedMemorySize, S_STAGES * S_STAGE_BYTES) != hipSuccess) return SS_ERR_HIP;
        attr_set = true;
    }
    const int tiles_o = (int)((O + BO - 1) / BO), tiles_t = (int)((M + BT - 1) / BT);
    hipLaunchKernelGGL(k_sparse_i8, dim3(tiles_o * tiles_t), dim3(G_THREADS), S_STAGES * S_STAGE_BYTES, static_cast<hipStream_t>(stream),
                       static_cast<const uint8_t*>(X_lifted), s_x, static_cast<const uint8_t*>(w_vals), static_cast<const uint8_t*>(w_meta), s_w,
                       M, O, K_lifted, static_cast<uint16_t*>(Y), ldy, tiles_o, tiles_t);
    return launch_status();
}

extern "C" const char* ss_status_string(ss_status s)
{
    switch (s) {
    case SS_OK: return "ok";
    case SS_ERR_NULL: return "null pointer";
    case SS_ERR_BAD_PATTERN_N: return "pattern parameter N outside 2..8";
    case SS_ERR_SHAPE: return "bad shape, stride or alignment";
    case SS_ERR_DTYPE: return "unsupported dtype";
    case SS_ERR_WORKSPACE: return "workspace";
    case SS_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" int slide_format_version(void) { return SS_FORMAT_VERSION; }
