// slide_sparse_gemm and dense_gemm for token counts between the decode regime and the point where
// 256 x 256 tiles fill the chip (roughly 64 < M <= 1024 on layers with a few thousand output channels).
//
// There the large-tile kernels leave most compute units idle (M = 256 on a 3584-channel layer is 14
// tiles for 256 units), so these kernels use 128 (one weight panel) x 128 (tokens) tiles, one tile per
// workgroup of four wavefronts, each wavefront accumulating 64 channels x 64 tokens (2 x 2 blocks of a
// 32x32 matrix instruction).  Operands go HBM/L2 -> LDS with direct-to-LDS loads into a ring of
// units of 128 k-bytes (all but one in flight while that one is computed: a lone workgroup on a compute
// unit is bound by load latency, so the ring is as deep as LDS allows; one barrier per unit); the inner
// loop is left to the compiler's scheduler: with at most a few tiles per compute unit the run time is
// set by how many units are busy, not by the last percent of matrix-core issue.
//   sparse: a unit is a 16 KB token tile plus the panel's 8 KB of stored values and 2 KB of index
//           words, which are already in operand-register order (packed_layout.h);
//   dense:  a unit is a 16 KB token tile plus a 16 KB tile of weight rows, both XOR-swizzled.
// The epilogue writes each lane's 16 consecutive channels of a token straight to Y.
#include "ss_common.h"
#include "packed_layout.h"
#include "mma_types.h"
#include "lds_pipe.h"
#include "device_info.h"

namespace ss {

constexpr int MD_WAVES = 4;
constexpr int MD_THREADS = 64 * MD_WAVES;
constexpr int MD_TILE = 128;                        // output channels and tokens per workgroup
constexpr int MD_S_RING = 3, MD_D_RING = 3;        // units of the operand rings (one computed, the others in flight)
constexpr int MD_ROWS_LOADS = MD_TILE / (8 * MD_WAVES);   // 8 rows per wavefront-wide load: 4 loads per wavefront and tile
constexpr int MD_TOK = MD_TILE * ROWB;              // 16 KB
constexpr int MD_AV = 8192, MD_AM = 2048;           // one unit of one panel: stored values, index words
constexpr int MD_S_UNIT = MD_TOK + MD_AV + MD_AM;   // 26 KB
constexpr int MD_D_UNIT = 2 * MD_TOK;               // 32 KB
constexpr int MD_S_LPU = MD_ROWS_LOADS + 2 + 1;     // direct loads per wavefront and unit
constexpr int MD_D_LPU = 2 * MD_ROWS_LOADS;
// fused lifting (6:8): a unit is a super-unit of 128 unlifted bytes = three steps of one panel
constexpr int MD_F_AV = 3 * 4096, MD_F_AM = 3 * 1024;
constexpr int MD_F_UNIT = MD_TOK + MD_F_AV + MD_F_AM;   // 31 KB
constexpr int MD_F_LPU = MD_ROWS_LOADS + 3 + 1;

// per-lane source offsets of the direct loads that fill a [128 x 128 B] swizzled tile; rows beyond the
// matrix are clamped to its last row (their products are never stored)
struct MidRowLoader {
    const uint8_t* base;                            // first row of the tile (wave-uniform)
    uint32_t off[MD_ROWS_LOADS];
    __device__ void init(const uint8_t* mat, int64_t ld, int64_t row0, int64_t nrows, int wave, int lane)
    {
        base = mat + row0 * ld;
        const int64_t left = nrows - row0;             // >= 1
        const int last = left > MD_TILE - 1 ? MD_TILE - 1 : (int)left - 1;
        const uint32_t ld32 = (uint32_t)ld;             // 128 rows x ld fits 32 bits (row bytes <= 2^23)
#pragma unroll
        for (int i = 0; i < MD_ROWS_LOADS; ++i) {
            const int row = (i * MD_WAVES + wave) * 8 + (lane >> 3);
            const int lc = (lane & 7) ^ swz(row);
            off[i] = (uint32_t)(row < last ? row : last) * ld32 + lc * 16;
        }
    }
    __device__ void issue(int64_t k0, uint8_t* lds_tile, int wave) const
    {
#pragma unroll
        for (int i = 0; i < MD_ROWS_LOADS; ++i) lds_dma16(base + k0, off[i], lds_tile + (i * MD_WAVES + wave) * 8 * ROWB);
    }
};

// acc[f][tb][r] of lane (n = lane & 31, h = lane >> 5) is channel o_wave + 64 h + 16 f + r of token t_wave + 32 tb + n
template <bool SCALED, typename ACC>
__device__ inline void mid_store(const ACC (&acc)[2][2], const float* __restrict__ s_x, const float* __restrict__ s_w, uint16_t* __restrict__ Y,
                                 int64_t ldy, int64_t M, int64_t O, int64_t o_wave, int64_t t_wave, int lane)
{
    const int n = lane & 31, h = lane >> 5;
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
            store_block16<SCALED>(acc[f][tb], s_x, s_w, Y, ldy, M, O, o_wave + 64 * h + 16 * f, t_wave + tb * 32 + n);
}

// Split k: the raw accumulators of k-range s of tile `tile` go to the workspace as
// ws[s][tile][wave][f][tb][register quad][lane] 16-byte groups (64 KB per tile and range, coalesced).
constexpr int MD_WS_TILE = MD_TILE * MD_TILE * 4;
template <typename ACC>
__device__ inline void mid_store_partial(const ACC (&acc)[2][2], void* ws, int64_t item, int wave, int lane)
{
    v4i* dst = static_cast<v4i*>(ws) + ((item * MD_WAVES + wave) * 16) * 64 + lane;
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                typedef decltype(acc[0][0][0] + acc[0][0][0]) elem_t;
                const elem_t q[4] = {acc[f][tb][4 * r4], acc[f][tb][4 * r4 + 1], acc[f][tb][4 * r4 + 2], acc[f][tb][4 * r4 + 3]};
                dst[((f * 2 + tb) * 4 + r4) * 64] = __builtin_bit_cast(v4i, q);
            }
}

// Sum of the S partial accumulators of every tile in range order (bit-reproducible also for fp32) and the
// scale epilogue.  One workgroup per (tile, wavefront of the GEMM kernel); thread (f, tb, register quad, lane) owns four
// consecutive channels of one token, so a range costs it one 16-byte load and up to eight ranges are in flight at once.
constexpr int MD_RED_THREADS = 1024;
template <int DT>
__global__ __launch_bounds__(MD_RED_THREADS) void k_mid_reduce(const v4i* __restrict__ ws, int S, int64_t ntiles, const float* __restrict__ s_x,
                                                               const float* __restrict__ s_w, int64_t M, int64_t O, uint16_t* __restrict__ Y,
                                                               int64_t ldy, int tiles_t)
{
    typedef Mma<DT> MM;
    typedef typename MM::acc_t acc_t;
    typedef decltype(acc_t{}[0] + acc_t{}[0]) elem_t;
    typedef elem_t quad_t __attribute__((ext_vector_type(4)));
    const int64_t tile = blockIdx.x / MD_WAVES;
    const int wave = blockIdx.x % MD_WAVES, wo = wave & 1, wt = wave >> 1;
    const int lane = threadIdx.x & 63, r4 = (threadIdx.x >> 6) & 3, ft = threadIdx.x >> 8, f = ft >> 1, tb = ft & 1;
    quad_t a = {0, 0, 0, 0};
    const v4i* src = ws + ((tile * MD_WAVES + wave) * 16 + ft * 4 + r4) * 64 + lane;
    const int64_t range_stride = ntiles * MD_WAVES * 16 * 64;             // 16-byte groups between consecutive k ranges
    int s = 0;
    for (; s + 8 <= S; s += 8) {
        quad_t q[8];
#pragma unroll
        for (int d = 0; d < 8; ++d) q[d] = __builtin_bit_cast(quad_t, src[(s + d) * range_stride]);
#pragma unroll
        for (int d = 0; d < 8; ++d) a += q[d];
    }
    if (s + 4 <= S) {
        quad_t q[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) q[d] = __builtin_bit_cast(quad_t, src[(s + d) * range_stride]);
#pragma unroll
        for (int d = 0; d < 4; ++d) a += q[d];
        s += 4;
    }
    {
        quad_t q[3];
#pragma unroll
        for (int d = 0; d < 3; ++d) q[d] = s + d < S ? __builtin_bit_cast(quad_t, src[(s + d) * range_stride]) : quad_t{0, 0, 0, 0};
#pragma unroll
        for (int d = 0; d < 3; ++d)
            if (s + d < S) a += q[d];
    }
    const int64_t panel = tile / tiles_t, t0 = (tile - panel * tiles_t) * MD_TILE;
    store_quad4<MM::SCALED>(a, s_x, s_w, Y, ldy, M, O, panel * PANEL + 32 * wo + 64 * (lane >> 5) + 16 * f + 4 * r4, t0 + wt * 64 + tb * 32 + (lane & 31));
}

// Tile of this workgroup.  Workgroup ids go round-robin over the 8 XCDs; when the tile count allows, the tiles are
// renumbered so that every XCD works on one contiguous run of tiles: the token tiles of a weight panel (consecutive
// tile numbers) then share that panel's weights in one L2 instead of fetching them once per XCD.
__device__ inline int mid_tile_of_block()
{
    const int nt = gridDim.x, b = blockIdx.x;
    return (nt & 7) == 0 ? (b & 7) * (nt >> 3) + (b >> 3) : b;
}

template <typename ACC> __device__ inline void mid_zero(ACC (&acc)[2][2])
{
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][tb][r] = 0;
}

// ---- sparse ---------------------------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(MD_THREADS) void k_sparse_mid(const uint8_t* __restrict__ XL, const float* __restrict__ s_x,
                                                           const uint8_t* __restrict__ w_vals, const uint8_t* __restrict__ w_meta,
                                                           const float* __restrict__ s_w, int64_t M, int64_t O, int64_t Kpb,
                                                           uint16_t* __restrict__ Y, int64_t ldy, int tiles_t, void* __restrict__ ws)
{
    typedef Mma<DT> MM;
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];     // MD_S_RING units
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wo = wave & 1, wt = wave >> 1;
    const int n = lane & 31, qb = lane >> 5;
    const int U_all = (int)(Kpb / (2 * FRAG_KB));
    // k range of this workgroup: units [u0, u0 + U); gridDim.y ranges, all non-empty (gridDim.y <= U_all)
    const int u0 = (int)((int64_t)blockIdx.y * U_all / gridDim.y), U = (int)((int64_t)(blockIdx.y + 1) * U_all / gridDim.y) - u0;
    const int tile = mid_tile_of_block();
    const int64_t panel = tile / tiles_t;
    const int64_t t0 = (int64_t)(tile - panel * tiles_t) * MD_TILE;

    MidRowLoader lb;
    lb.init(XL + (int64_t)u0 * ROWB, Kpb, t0, M, wave, lane);
    // unit u of the panel: 8 KB of values [step 2][fragment 4][lane 64][16 B], 2 KB of index words
    // [step 2][lane 64][fragment 4][4 B]; wavefront w copies value pieces 2w, 2w + 1 (1 KB each) and index piece w & 1
    const uint8_t* av_src = w_vals + (panel * U_all + u0) * MD_AV + wave * 2048;
    const uint8_t* am_src = w_meta + (panel * U_all + u0) * MD_AM + (wave & 1) * 1024;
    const uint32_t lane16 = lane * 16;
    auto issue = [&](int u, int slot) {
        uint8_t* st = smem + slot * MD_S_UNIT;
        lb.issue((int64_t)u * ROWB, st, wave);
        lds_dma16(av_src + (int64_t)u * MD_AV, lane16, st + MD_TOK + wave * 2048);
        lds_dma16(av_src + (int64_t)u * MD_AV + 1024, lane16, st + MD_TOK + wave * 2048 + 1024);
        lds_dma16(am_src + (int64_t)u * MD_AM, lane16, st + MD_TOK + MD_AV + (wave & 1) * 1024);
    };

    typename MM::acc_t acc[2][2];
    mid_zero(acc);
    constexpr int AHEAD = MD_S_RING - 1;                                 // units requested ahead of the one being computed
#pragma unroll
    for (int i = 0; i < AHEAD; ++i)
        if (i < U) issue(i, i);
    int slot = 0, lslot = AHEAD;
    for (int u = 0; u < U; ++u) {
        // own loads of unit u have landed (the AHEAD - 1 units behind it may still be in flight; at the end of
        // the k range everything is awaited at once), own reads of unit u-1 have returned
        if (u + AHEAD <= U) wait_vmcnt<(AHEAD - 1) * MD_S_LPU>(); else wait_vmcnt<0>();
        wg_barrier();                                                    // ... for every wavefront
        if (u + AHEAD < U) issue(u + AHEAD, lslot);                      // into the slot of unit u-1
        const uint8_t* st = smem + slot * MD_S_UNIT;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            v4i a[2]; v8i b[2];
            typedef int v2i __attribute__((ext_vector_type(2)));
            const v2i idx = *reinterpret_cast<const v2i*>(st + MD_TOK + MD_AV + (h * 64 + lane) * 16 + wo * 8);
#pragma unroll
            for (int f = 0; f < 2; ++f) a[f] = *reinterpret_cast<const v4i*>(st + MD_TOK + ((h * 4 + 2 * wo + f) * 64 + lane) * 16);
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int row = wt * 64 + tb * 32 + n;
                const v4i lo = *tile_chunk(st, row, 4 * h + 2 * qb), hi = *tile_chunk(st, row, 4 * h + 2 * qb + 1);
                b[tb] = (v8i){lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) acc[f][tb] = MM::sparse(a[f], b[tb], acc[f][tb], idx[f]);
        }
        slot = slot == MD_S_RING - 1 ? 0 : slot + 1;
        lslot = lslot == MD_S_RING - 1 ? 0 : lslot + 1;
    }
    if (gridDim.y > 1) mid_store_partial(acc, ws, (int64_t)blockIdx.y * gridDim.x + tile, wave, lane);
    else mid_store<MM::SCALED>(acc, s_x, s_w, Y, ldy, M, O, panel * PANEL + 32 * wo, t0 + wt * 64, lane);
}

// ---- sparse, lifting applied in the operand read (6:8, weights packed by slide_decompose_fused) --------------
// Same tile and ring as k_sparse_mid, but the token tile holds UNLIFTED rows (a super-unit of 128 bytes per row and
// unit, as in the dense kernel) and a unit is three matrix-instruction steps deep: B lane (n, qb) reads the 64 bytes
// [64 qb, 64 qb + 64) of its row as 16 registers, uses the first eight in step 0, the second eight in step 1 and builds
// the eight middle windows of step 2 in registers (packed_layout.h, fused_window).  The k loop is as long as the
// dense kernel's, with three sparse instructions where that one issues four dense ones.
template <int DT, int RING>
__global__ __launch_bounds__(MD_THREADS) void k_sparse_fused_mid(const uint8_t* __restrict__ Xq, const float* __restrict__ s_x,
                                                                 const uint8_t* __restrict__ w_vals, const uint8_t* __restrict__ w_meta,
                                                                 const float* __restrict__ s_w, int64_t M, int64_t O, int U_all, int64_t ldxb,
                                                                 uint16_t* __restrict__ Y, int64_t ldy, int tiles_t, void* __restrict__ ws)
{
    typedef Mma<DT> MM;
    constexpr int ES = MM::ES;
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];     // RING units
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wo = wave & 1, wt = wave >> 1;
    const int n = lane & 31, qb = lane >> 5;
    const int u0 = (int)((int64_t)blockIdx.y * U_all / gridDim.y), U = (int)((int64_t)(blockIdx.y + 1) * U_all / gridDim.y) - u0;
    const int tile = mid_tile_of_block();
    const int64_t panel = tile / tiles_t;
    const int64_t t0 = (int64_t)(tile - panel * tiles_t) * MD_TILE;

    MidRowLoader lb;
    lb.init(Xq + (int64_t)u0 * ROWB, ldxb, t0, M, wave, lane);
    // super-unit u of the panel: 12 KB of values [step 3][fragment 4][lane 64][16 B], 3 KB of index words
    // [step 3][lane 64][fragment 4][4 B]; wavefront w copies value pieces 3w .. 3w + 2 (1 KB each) and 768 bytes
    // of the index words (lanes 0..47 of one load)
    const uint8_t* av_src = w_vals + (panel * U_all + u0) * MD_F_AV + wave * 3072;
    const uint8_t* am_src = w_meta + (panel * U_all + u0) * MD_F_AM + wave * 768;
    const uint32_t lane16 = lane * 16;
    auto issue = [&](int u, int slot) {
        uint8_t* st = smem + slot * MD_F_UNIT;
        lb.issue((int64_t)u * ROWB, st, wave);
#pragma unroll
        for (int i = 0; i < 3; ++i) lds_dma16(av_src + (int64_t)u * MD_F_AV + i * 1024, lane16, st + MD_TOK + wave * 3072 + i * 1024);
        if (lane < 48) lds_dma16(am_src + (int64_t)u * MD_F_AM, lane16, st + MD_TOK + MD_F_AV + wave * 768);
    };

    typename MM::acc_t acc[2][2];
    mid_zero(acc);
    constexpr int AHEAD = RING - 1;
#pragma unroll
    for (int i = 0; i < AHEAD; ++i)
        if (i < U) issue(i, i);
    int slot = 0, lslot = AHEAD;
    for (int u = 0; u < U; ++u) {
        if (u + AHEAD <= U) wait_vmcnt<(AHEAD - 1) * MD_F_LPU>(); else wait_vmcnt<0>();
        wg_barrier();
        if (u + AHEAD < U) issue(u + AHEAD, lslot);
        const uint8_t* st = smem + slot * MD_F_UNIT;
        // the lane's 64 unlifted bytes of both token blocks
        int x[2][16];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            const int row = wt * 64 + tb * 32 + n;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const v4i v = *tile_chunk(st, row, 4 * qb + c);
#pragma unroll
                for (int e = 0; e < 4; ++e) x[tb][4 * c + e] = v[e];
            }
        }
#pragma unroll
        for (int J = 0; J < 3; ++J) {
            v4i a[2]; v8i b[2];
            typedef int v2i __attribute__((ext_vector_type(2)));
            const v2i idx = *reinterpret_cast<const v2i*>(st + MD_TOK + MD_F_AV + (J * 64 + lane) * 16 + wo * 8);
#pragma unroll
            for (int f = 0; f < 2; ++f) a[f] = *reinterpret_cast<const v4i*>(st + MD_TOK + ((J * 4 + 2 * wo + f) * 64 + lane) * 16);
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int jd = 0; jd < 8; ++jd) {
                    if (J < 2) b[tb][jd] = x[tb][8 * J + jd];
                    else if constexpr (ES == 1) b[tb][jd] = (int)__builtin_amdgcn_alignbyte((uint32_t)x[tb][2 * jd + 1], (uint32_t)x[tb][2 * jd], 2);
                    else b[tb][jd] = x[tb][4 * (jd >> 1) + 1 + (jd & 1)];
                }
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) acc[f][tb] = MM::sparse(a[f], b[tb], acc[f][tb], idx[f]);
        }
        slot = slot == RING - 1 ? 0 : slot + 1;
        lslot = lslot == RING - 1 ? 0 : lslot + 1;
    }
    if (gridDim.y > 1) mid_store_partial(acc, ws, (int64_t)blockIdx.y * gridDim.x + tile, wave, lane);
    else mid_store<MM::SCALED>(acc, s_x, s_w, Y, ldy, M, O, panel * PANEL + 32 * wo, t0 + wt * 64, lane);
}

// ---- dense ----------------------------------------------------------------------------------------------
template <int DT, int RING>
__global__ __launch_bounds__(MD_THREADS) void k_dense_mid(const uint8_t* __restrict__ Xq, const float* __restrict__ s_x, const uint8_t* __restrict__ Wq,
                                                          const float* __restrict__ s_w, int64_t M, int64_t O, int64_t Kb, uint16_t* __restrict__ Y,
                                                          int64_t ldy, int tiles_t, void* __restrict__ ws)
{
    typedef Mma<DT> MM;
    typedef typename MM::dfrag_t frag_t;
    constexpr int SUB = MM::DENSE_SUB, NSUB = ROWB / SUB, RPF = SUB / 32;    // k-bytes per instruction, instructions per unit, 16-byte reads per fragment
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wo = wave & 1, wt = wave >> 1;
    const int row = lane & 31, q = lane >> 5;
    const int U_all = (int)(Kb / ROWB);
    const int u0 = (int)((int64_t)blockIdx.y * U_all / gridDim.y), U = (int)((int64_t)(blockIdx.y + 1) * U_all / gridDim.y) - u0;
    const int tile = mid_tile_of_block();
    const int64_t panel = tile / tiles_t;
    const int64_t t0 = (int64_t)(tile - panel * tiles_t) * MD_TILE;

    MidRowLoader la, lb;
    la.init(Wq + (int64_t)u0 * ROWB, Kb, panel * PANEL, O, wave, lane);
    lb.init(Xq + (int64_t)u0 * ROWB, Kb, t0, M, wave, lane);
    auto issue = [&](int u, int slot) {
        la.issue((int64_t)u * ROWB, smem + slot * MD_D_UNIT, wave);
        lb.issue((int64_t)u * ROWB, smem + slot * MD_D_UNIT + MD_TOK, wave);
    };
    // rows of the weight fragments in panel order, so that a lane's accumulators are consecutive channels
    int arow[2], brow[2];
#pragma unroll
    for (int f = 0; f < 2; ++f) arow[f] = panel_row(2 * wo + f, row);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) brow[tb] = wt * 64 + tb * 32 + row;

    typename MM::acc_t acc[2][2];
    mid_zero(acc);
    constexpr int AHEAD = RING - 1;
#pragma unroll
    for (int i = 0; i < AHEAD; ++i)
        if (i < U) issue(i, i);
    int slot = 0, lslot = AHEAD;
    for (int u = 0; u < U; ++u) {
        if (u + AHEAD <= U) wait_vmcnt<(AHEAD - 1) * MD_D_LPU>(); else wait_vmcnt<0>();
        wg_barrier();
        if (u + AHEAD < U) issue(u + AHEAD, lslot);
        const uint8_t* sa = smem + slot * MD_D_UNIT;
        const uint8_t* sb = sa + MD_TOK;
#pragma unroll
        for (int t = 0; t < NSUB; ++t) {
            frag_t a[2], b[2];
#pragma unroll
            for (int piece = 0; piece < RPF; ++piece) {
                const int lc = t * (SUB / 16) + q * RPF + piece;
#pragma unroll
                for (int f = 0; f < 2; ++f) {
                    const v4i v = *tile_chunk(sa, arow[f], lc);
#pragma unroll
                    for (int e = 0; e < 4; ++e) a[f][4 * piece + e] = v[e];
                }
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    const v4i v = *tile_chunk(sb, brow[tb], lc);
#pragma unroll
                    for (int e = 0; e < 4; ++e) b[tb][4 * piece + e] = v[e];
                }
            }
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) acc[f][tb] = MM::dense(a[f], b[tb], acc[f][tb]);
        }
        slot = slot == RING - 1 ? 0 : slot + 1;
        lslot = lslot == RING - 1 ? 0 : lslot + 1;
    }
    if (gridDim.y > 1) mid_store_partial(acc, ws, (int64_t)blockIdx.y * gridDim.x + tile, wave, lane);
    else mid_store<MM::SCALED>(acc, s_x, s_w, Y, ldy, M, O, panel * PANEL + 32 * wo, t0 + wt * 64, lane);
}

}  // namespace ss

using namespace ss;

template <int DT>
static ss_status launch_mid_reduce(const void* ws, int S, int64_t ntiles, const float* s_x, const float* s_w, int64_t M, int64_t O, void* Y,
                                   int64_t ldy, int tiles_t, hipStream_t stream)
{
    hipLaunchKernelGGL((k_mid_reduce<DT>), dim3((unsigned)(ntiles * MD_WAVES)), dim3(MD_RED_THREADS), 0, stream, static_cast<const v4i*>(ws), S, ntiles,
                       s_x, s_w, M, O, static_cast<uint16_t*>(Y), ldy, tiles_t);
    return launch_status();
}

template <int DT>
static ss_status launch_sparse_mid_dt(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M,
                                      int64_t O, int64_t Kpb, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream)
{
    const int tiles_t = (int)((M + MD_TILE - 1) / MD_TILE);
    const int64_t ntiles = (O + PANEL - 1) / PANEL * tiles_t;
    constexpr int lds = MD_S_RING * MD_S_UNIT;
    if (allow_dynamic_lds<k_sparse_mid<DT>>(lds) != SS_OK) return SS_ERR_HIP;
    hipLaunchKernelGGL((k_sparse_mid<DT>), dim3((unsigned)ntiles, (unsigned)S), dim3(MD_THREADS), lds, stream, static_cast<const uint8_t*>(XL), s_x,
                       static_cast<const uint8_t*>(w_vals), static_cast<const uint8_t*>(w_meta), s_w, M, O, Kpb, static_cast<uint16_t*>(Y), ldy,
                       tiles_t, ws);
    if (launch_status() != SS_OK) return SS_ERR_HIP;
    return S > 1 ? launch_mid_reduce<DT>(ws, S, ntiles, s_x, s_w, M, O, Y, ldy, tiles_t, stream) : SS_OK;
}

template <int DT, int RING>
static ss_status launch_sparse_fused_mid_ring(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M,
                                              int64_t O, int U, int64_t ldxb, void* Y, int64_t ldy, void* ws, int S, int tiles_t, int64_t ntiles,
                                              hipStream_t stream)
{
    constexpr int lds = RING * MD_F_UNIT;
    if (allow_dynamic_lds<k_sparse_fused_mid<DT, RING>>(lds) != SS_OK) return SS_ERR_HIP;
    hipLaunchKernelGGL((k_sparse_fused_mid<DT, RING>), dim3((unsigned)ntiles, (unsigned)S), dim3(MD_THREADS), lds, stream,
                       static_cast<const uint8_t*>(Xq), s_x, static_cast<const uint8_t*>(w_vals), static_cast<const uint8_t*>(w_meta), s_w, M, O, U,
                       ldxb, static_cast<uint16_t*>(Y), ldy, tiles_t, ws);
    return launch_status();
}

template <int DT>
static ss_status launch_sparse_fused_mid_dt(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M,
                                            int64_t O, int U, int64_t ldxb, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream)
{
    const int tiles_t = (int)((M + MD_TILE - 1) / MD_TILE);
    const int64_t ntiles = (O + PANEL - 1) / PANEL * tiles_t;
    // Ring depth: with more workgroups than compute units a ring of two units (62 KB) lets two workgroups share a
    // unit's LDS and cover each other's load latency; otherwise a lone workgroup gets the deeper ring.
    // (measured, INT8: 3584 -> 37888 at M = 128, 296 workgroups: 42 -> 30 us; 3584 -> 4608 at M = 1024: 42 -> 29 us;
    // 18944 -> 3584 at M = 1024, 224 workgroups: 105 us with two units, 95 with three, 92 with four)
    const ss_status st = ntiles * S > cu_count()
        ? launch_sparse_fused_mid_ring<DT, 2>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, tiles_t, ntiles, stream)
        : launch_sparse_fused_mid_ring<DT, 4>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, tiles_t, ntiles, stream);
    if (st != SS_OK) return st;
    return S > 1 ? launch_mid_reduce<DT>(ws, S, ntiles, s_x, s_w, M, O, Y, ldy, tiles_t, stream) : SS_OK;
}

template <int DT, int RING>
static ss_status launch_dense_mid_ring(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, void* Y,
                                       int64_t ldy, void* ws, int S, int tiles_t, int64_t ntiles, hipStream_t stream)
{
    constexpr int lds = RING * MD_D_UNIT;
    if (allow_dynamic_lds<k_dense_mid<DT, RING>>(lds) != SS_OK) return SS_ERR_HIP;
    hipLaunchKernelGGL((k_dense_mid<DT, RING>), dim3((unsigned)ntiles, (unsigned)S), dim3(MD_THREADS), lds, stream, static_cast<const uint8_t*>(Xq),
                       s_x, static_cast<const uint8_t*>(Wq), s_w, M, O, Kb, static_cast<uint16_t*>(Y), ldy, tiles_t, ws);
    return launch_status();
}

template <int DT>
static ss_status launch_dense_mid_dt(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, void* Y,
                                     int64_t ldy, void* ws, int S, hipStream_t stream)
{
    const int tiles_t = (int)((M + MD_TILE - 1) / MD_TILE);
    const int64_t ntiles = (O + PANEL - 1) / PANEL * tiles_t;
    // ring depth as for the fused sparse kernel: two units (64 KB) where two workgroups can share a compute unit
    const ss_status st = ntiles * S > cu_count()
        ? launch_dense_mid_ring<DT, 2>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, tiles_t, ntiles, stream)
        : launch_dense_mid_ring<DT, MD_D_RING>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, tiles_t, ntiles, stream);
    if (st != SS_OK) return st;
    return S > 1 ? launch_mid_reduce<DT>(ws, S, ntiles, s_x, s_w, M, O, Y, ldy, tiles_t, stream) : SS_OK;
}

// Host side, called by the C entry points.  Arguments are already validated.
namespace ss {

// Number of k ranges for ntiles 128 x 128 tiles over `units` 128-byte k units with a workspace of ws_bytes:
// about one workgroup per compute unit, at least eight units per range, no more than the workspace holds
// (measured on 3584 -> 4608 at M = 128: 22 us unsplit, 15 us with 4 to 6 ranges, 17 us with 8).
int mid_splits(int64_t M, int64_t O, int64_t units, size_t ws_bytes)
{
    const int64_t ntiles = mid_tiles(M, O);
    int64_t S = cu_count() / ntiles;
    if (S > units / 8) S = units / 8;
    const int64_t fit = (int64_t)(ws_bytes / ((size_t)ntiles * MD_WS_TILE));
    if (S > fit) S = fit;
    return S < 2 ? 1 : (int)S;
}

size_t mid_workspace_bytes(int64_t M, int64_t O, int S)
{
    return S > 1 ? (size_t)S * mid_tiles(M, O) * MD_WS_TILE : 0;
}

ss_status launch_sparse_mid(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                            int64_t Kpb, ss_dtype dtype, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream)
{
    switch (dtype) {
    case SS_I8: return launch_sparse_mid_dt<SS_I8>(XL, s_x, w_vals, w_meta, s_w, M, O, Kpb, Y, ldy, ws, S, stream);
    case SS_FP8_E4M3: return launch_sparse_mid_dt<SS_FP8_E4M3>(XL, s_x, w_vals, w_meta, s_w, M, O, Kpb, Y, ldy, ws, S, stream);
    case SS_BF16: return launch_sparse_mid_dt<SS_BF16>(XL, s_x, w_vals, w_meta, s_w, M, O, Kpb, Y, ldy, ws, S, stream);
    case SS_FP16: return launch_sparse_mid_dt<SS_FP16>(XL, s_x, w_vals, w_meta, s_w, M, O, Kpb, Y, ldy, ws, S, stream);
    }
    return SS_ERR_DTYPE;
}

ss_status launch_sparse_fused_mid(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                                  int U, int64_t ldxb, ss_dtype dtype, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream)
{
    switch (dtype) {
    case SS_I8: return launch_sparse_fused_mid_dt<SS_I8>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, stream);
    case SS_FP8_E4M3: return launch_sparse_fused_mid_dt<SS_FP8_E4M3>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, stream);
    case SS_BF16: return launch_sparse_fused_mid_dt<SS_BF16>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, stream);
    case SS_FP16: return launch_sparse_fused_mid_dt<SS_FP16>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, stream);
    }
    return SS_ERR_DTYPE;
}

ss_status launch_dense_mid(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, ss_dtype dtype,
                           void* Y, int64_t ldy, void* ws, int S, hipStream_t stream)
{
    switch (dtype) {
    case SS_I8: return launch_dense_mid_dt<SS_I8>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, stream);
    case SS_FP8_E4M3: return launch_dense_mid_dt<SS_FP8_E4M3>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, stream);
    case SS_BF16: return launch_dense_mid_dt<SS_BF16>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, stream);
    case SS_FP16: return launch_dense_mid_dt<SS_FP16>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, stream);
    }
    return SS_ERR_DTYPE;
}

}  // namespace ss
