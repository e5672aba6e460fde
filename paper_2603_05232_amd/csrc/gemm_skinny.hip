// slide_sparse_gemm and dense_gemm for few tokens (M <= 64): the decode regime, bound by streaming the
// weights from HBM once, not by the matrix cores.
//
// A workgroup of four wavefronts owns FPW x 32 output channels (FPW matrix-instruction fragments, FPW = 1, 2
// or 4: as many as still leave at least one workgroup per compute unit) and all tokens; the wavefronts (4,
// or 8 when there are fewer workgroups than compute units) split the k range by units of 128 bytes of a row
// (unit u goes to wavefront u mod the number of wavefronts), so every workgroup is
// four independent load streams, enough of them in flight on every compute unit to keep the memory system
// busy.  More fragments per workgroup mean fewer re-reads of the token rows (sparse kernel only: the dense
// kernel's LDS staging makes one fragment per workgroup the faster choice).  Operands go from global memory
// straight into registers (a ring of two to four units per wavefront, all in flight); partial sums of the wavefronts meet
// in LDS in a fixed order (bit-reproducible also for fp32 accumulators) and wavefront 0 applies the scale epilogue.
// With a workspace the k range is also split over workgroups (gridDim.y ranges) and k_skinny_reduce adds their partial
// sums in range order.
//   sparse: the packed weights are already in operand-register order, 16 bytes + one index word per lane and
//           step, fully coalesced; no LDS in the main loop.
//           The same kernel serves the fused path (6:8, unlifted tokens, weights packed by slide_decompose_fused): a unit
//           is then three steps deep and the lifted B operands are built in registers.
//   dense:  row-major weights are fetched as whole 128-byte lines (8 rows per load instruction) and turned
//           into fragments through a wavefront-private 4 KB LDS tile.
// Tokens are the B operand, read directly from the L2-resident activation rows (whole lines per unit).
#include "ss_common.h"
#include "packed_layout.h"
#include "mma_types.h"
#include "device_info.h"
#include <cstdlib>

namespace ss {

// wavefronts per workgroup: 4, or 8 when there are fewer workgroups than compute units (more load streams per unit)

// units a wavefront keeps in flight in registers: 4 where a workgroup is a single fragment (few workgroups, each
// wavefront a chain of load round trips), 2 where it holds several fragments (many workgroups per compute unit)
template <int FPW, int TB> constexpr int SK_DEPTH = FPW == 1 ? (TB == 1 ? 4 : 3) : 2;

template <typename ACC> __device__ inline void sk_zero(ACC& a)
{
#pragma unroll
    for (int r = 0; r < 16; ++r) a[r] = 0;
}

// Sum of the wavefronts' partial accumulators, in wavefront order, returned in wavefront 0.
template <int SK_WAVES, typename ACC, int TB>
__device__ inline void sk_reduce(ACC (&acc)[TB], uint8_t* red, int wave, int lane)
{
    // red: [wave 1..][accumulator][reg 16][lane 64] 4-byte words
    typedef decltype(acc[0][0] + acc[0][0]) elem_t;
    elem_t* r = reinterpret_cast<elem_t*>(red);
    if (wave > 0) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int i = 0; i < 16; ++i) r[(((wave - 1) * TB + tb) * 16 + i) * 64 + lane] = acc[tb][i];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int w = 1; w < SK_WAVES; ++w)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tb][i] += r[(((w - 1) * TB + tb) * 16 + i) * 64 + lane];
    }
}

// Epilogue of one wavefront: acc[tb][r] of lane (n = lane & 31, hh = lane >> 5) is channel o_lane + r of token
// 32 tb + n, with o_lane the first of the lane's 16 consecutive channels.
template <bool SCALED, typename ACC, int TB>
__device__ inline void sk_store(const ACC (&acc)[TB], const float* __restrict__ s_x, const float* __restrict__ s_w, uint16_t* __restrict__ Y,
                                int64_t ldy, int64_t M, int64_t O, int64_t o_lane, int lane)
{
    const int n = lane & 31;
    float sw[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        sw[i] = 1.0f;
        if constexpr (SCALED) { const int64_t o = o_lane + i; sw[i] = s_w[o < O ? o : O - 1]; }
    }
    const bool vec_ok = ((ldy & 7) == 0) && (((uintptr_t)Y & 15) == 0) && ((o_lane & 7) == 0) && o_lane + 16 <= O;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int64_t tok = tb * 32 + n;
        if (tok >= M) continue;
        float sx = 1.0f;
        if constexpr (SCALED) sx = s_x[tok];
        uint32_t w[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            if constexpr (SCALED) w[q] = pack_bf16x2(((float)acc[tb][2 * q] * sx) * sw[2 * q], ((float)acc[tb][2 * q + 1] * sx) * sw[2 * q + 1]);
            else w[q] = pack_bf16x2((float)acc[tb][2 * q], (float)acc[tb][2 * q + 1]);
        }
        uint16_t* dst = Y + tok * ldy + o_lane;
        if (vec_ok) {
            reinterpret_cast<uint4*>(dst)[0] = make_uint4(w[0], w[1], w[2], w[3]);
            reinterpret_cast<uint4*>(dst)[1] = make_uint4(w[4], w[5], w[6], w[7]);
        } else {
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (o_lane + e < O) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
        }
    }
}

// Split k: the raw accumulators of k range blockIdx.y of workgroup column `col` (0 .. gridDim.x - 1) go to the workspace as
// ws[range][column][accumulator][register quad][lane] 16-byte groups.
template <typename ACC, int NACC>
__device__ inline void sk_store_partial(const ACC (&acc)[NACC], void* ws, int col, int lane)
{
    typedef decltype(acc[0][0] + acc[0][0]) elem_t;
    v4i* dst = static_cast<v4i*>(ws) + (((int64_t)blockIdx.y * gridDim.x + col) * NACC * 4) * 64 + lane;
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const elem_t q[4] = {acc[i][4 * r4], acc[i][4 * r4 + 1], acc[i][4 * r4 + 2], acc[i][4 * r4 + 3]};
            dst[(i * 4 + r4) * 64] = __builtin_bit_cast(v4i, q);
        }
}

// ---- sparse ---------------------------------------------------------------------------------------------
// Operands of one unit of one wavefront.  Lifted input: a unit is 128 lifted bytes = NS = 2 steps of 64 lifted bytes.
// FUSED (6:8, unlifted input, weights packed by slide_decompose_fused): a unit is a super-unit of 128 unlifted bytes
// = NS = 3 steps; B lane (n, qb) loads the 64 bytes [64 qb, 64 qb + 64) of its token's super-unit, uses the first
// 32 in step 0, the second 32 in step 1 and builds the eight middle windows of step 2 in registers
// (packed_layout.h, fused_window): the k loop is as long as the dense kernel's and the token rows are read once,
// not 1.5 times.
template <int TB, int FPW, int NS> struct SkSparseUnit { v4i a[NS][FPW]; int idx[NS][FPW]; v4i b[TB][4]; };

template <int DT, int TB, int FPW, int SK_WAVES, bool FUSED>
__global__ __launch_bounds__(64 * SK_WAVES) void k_sparse_skinny(const uint8_t* __restrict__ XL, const float* __restrict__ s_x,
                                                               const uint8_t* __restrict__ w_vals, const uint8_t* __restrict__ w_meta,
                                                               const float* __restrict__ s_w, int64_t M, int64_t O, int U, int64_t ldxb,
                                                               uint16_t* __restrict__ Y, int64_t ldy, void* __restrict__ ws)
{
    typedef Mma<DT> MM;
    typedef int idx_t __attribute__((ext_vector_type(FPW)));
    constexpr int NS = FUSED ? 3 : 2;                   // steps per unit
    __shared__ __attribute__((aligned(16))) uint8_t red[(SK_WAVES - 1) * FPW * TB * 16 * 64 * 4];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    constexpr int GROUPS = FRAGS_PER_PANEL / FPW;       // workgroups per panel
    // Workgroup -> (panel, fragment group).  Workgroup ids go round-robin over the 8 XCDs; the GROUPS workgroups of a panel
    // read the same index-word lines (4 bytes per lane and fragment out of 16) and the same token rows, so they are placed
    // on one XCD, where the second to fourth of them hit in its L2 (single-fragment workgroups on 3584 -> 4608 fetched
    // 25 MB for 15.6 MB of packed weights before).  Panels beyond the last whole group of eight keep the plain order.
    int col = blockIdx.x;
    if (GROUPS > 1 && ((gridDim.x & 7) == 0 || gridDim.y == 1)) {      // workgroup id mod 8 == blockIdx.x mod 8
        const int whole = (int)(gridDim.x / (8 * GROUPS)) * (8 * GROUPS);
        if (col < whole) { const int xcd = col & 7, j = col >> 3; col = ((j / GROUPS) * 8 + xcd) * GROUPS + j % GROUPS; }
    }
    const int64_t panel = col / GROUPS;
    const int f0 = (col % GROUPS) * FPW;                // first fragment of this workgroup
    // values [panel][step][fragment][lane] 16 B, index words [panel][step][lane][fragment] 4 B
    const v4i* av = reinterpret_cast<const v4i*>(w_vals) + (panel * NS * U * FRAGS_PER_PANEL + f0) * 64 + lane;
    const int* am = reinterpret_cast<const int*>(w_meta) + (panel * NS * U * 64 + lane) * FRAGS_PER_PANEL + f0;
    // token rows: lane (n, qb) holds the bytes [32 qb, 32 qb + 32) of token n within a step (lifted input) or
    // [64 qb, 64 qb + 64) within a super-unit (unlifted input)
    // Lanes whose token does not exist load nothing (their products are never stored): a load instruction costs the
    // memory pipeline by its active lanes, and with a single token 31 of 32 would fetch copies.
    const uint8_t* xb[TB];
    bool live[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        int64_t tok = tb * 32 + (lane & 31);
        live[tb] = tok < M;
        tok = live[tb] ? tok : M - 1;
        xb[tb] = XL + tok * ldxb + (FUSED ? 64 : 32) * (lane >> 5);
    }
    auto load = [&](SkSparseUnit<TB, FPW, NS>& R, int u) {
#pragma unroll
        for (int h = 0; h < NS; ++h) {
            const int64_t s = NS * (int64_t)u + h;
#pragma unroll
            for (int f = 0; f < FPW; ++f) R.a[h][f] = av[s * (FRAGS_PER_PANEL * 64) + f * 64];
            if constexpr (FPW == 1) R.idx[h][0] = am[s * (64 * FRAGS_PER_PANEL)];
            else {
                const idx_t w = *reinterpret_cast<const idx_t*>(am + s * (64 * FRAGS_PER_PANEL));   // one load for all fragments
#pragma unroll
                for (int f = 0; f < FPW; ++f) R.idx[h][f] = w[f];
            }
        }
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
            if (live[tb]) {
                if constexpr (FUSED) {
                    const v4i* p = reinterpret_cast<const v4i*>(xb[tb] + (int64_t)u * KSTEP);
#pragma unroll
                    for (int c = 0; c < 4; ++c) R.b[tb][c] = p[c];
                } else {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const v4i* p = reinterpret_cast<const v4i*>(xb[tb] + (2 * (int64_t)u + h) * FRAG_KB);
                        R.b[tb][2 * h] = p[0];
                        R.b[tb][2 * h + 1] = p[1];
                    }
                }
            }
    };
    // B operand of step h from the unit's token registers
    auto operand = [&](const v4i (&x)[4], int h) -> v8i {
        if (!FUSED || h < 2) {
            const v4i lo = x[2 * h], hi = x[2 * h + 1];
            return v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
        v8i b;
#pragma unroll
        for (int jd = 0; jd < 8; ++jd) {
            if constexpr (MM::ES == 1) {                 // bytes 2..5 of block jd (registers 2 jd, 2 jd + 1)
                const int r0 = 2 * jd, r1 = 2 * jd + 1;
                b[jd] = (int)__builtin_amdgcn_alignbyte((uint32_t)x[r1 >> 2][r1 & 3], (uint32_t)x[r0 >> 2][r0 & 3], 2);
            } else {                                     // elements 2..5 of block jd >> 1: its registers 1 and 2
                const int r = 4 * (jd >> 1) + 1 + (jd & 1);
                b[jd] = x[r >> 2][r & 3];
            }
        }
        return b;
    };
    typename MM::acc_t acc[FPW * TB];
#pragma unroll
    for (int i = 0; i < FPW * TB; ++i) sk_zero(acc[i]);
    // A wavefront's units go through a ring of D register stages, all of them in flight: a lone wavefront's chain of
    // load round trips (a few units, each a trip to HBM) is what bounds the kernel where workgroups are single fragments.
    constexpr int D = SK_DEPTH<FPW, TB>;
    SkSparseUnit<TB, FPW, NS> st[D];
#pragma unroll
    for (int d = 0; d < D; ++d)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int j = 0; j < 4; ++j) st[d].b[tb][j] = v4i{0, 0, 0, 0};     // lanes without a token keep zeros
    // k range of this workgroup: units [u, u_end) of U; gridDim.y ranges
    const int u_end = (int)((int64_t)(blockIdx.y + 1) * U / gridDim.y);
    const int u0 = (int)((int64_t)blockIdx.y * U / gridDim.y) + wave;
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (u0 + d * SK_WAVES < u_end) load(st[d], u0 + d * SK_WAVES);
    for (int u = u0; u < u_end; u += D * SK_WAVES) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int uu = u + d * SK_WAVES;
            if (uu < u_end) {
#pragma unroll
                for (int h = 0; h < NS; ++h)
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) {
                        const v8i b = operand(st[d].b[tb], h);
#pragma unroll
                        for (int f = 0; f < FPW; ++f) acc[f * TB + tb] = MM::sparse(st[d].a[h][f], b, acc[f * TB + tb], st[d].idx[h][f]);
                    }
                if (uu + D * SK_WAVES < u_end) load(st[d], uu + D * SK_WAVES);
            }
        }
    }
    sk_reduce<SK_WAVES, typename MM::acc_t, FPW * TB>(acc, red, wave, lane);
    if (wave == 0) {
        if (gridDim.y > 1) { sk_store_partial<typename MM::acc_t, FPW * TB>(acc, ws, col, lane); return; }
#pragma unroll
        for (int f = 0; f < FPW; ++f) {
            typename MM::acc_t part[TB];
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) part[tb] = acc[f * TB + tb];
            sk_store<MM::SCALED, typename MM::acc_t, TB>(part, s_x, s_w, Y, ldy, M, O, panel * PANEL + 64 * (lane >> 5) + 16 * (f0 + f), lane);
        }
    }
}

// ---- dense ----------------------------------------------------------------------------------------------
// Row i (0..31) of a weight fragment is output channel o0 + 16 ((i >> 2) & 1) + 4 (i >> 3) + (i & 3), which
// makes the 16 accumulator registers of a lane 16 consecutive channels (the same idea as inside a packed panel).
__device__ inline int sk_frag_row(int i) { return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3); }

template <int TB, int FPW> struct SkDenseUnit { v4i a[FPW][4]; v4i b[TB][4]; };

template <int DT, int TB, int FPW, int SK_WAVES>
__global__ __launch_bounds__(64 * SK_WAVES) void k_dense_skinny(const uint8_t* __restrict__ Xq, const float* __restrict__ s_x,
                                                              const uint8_t* __restrict__ Wq, const float* __restrict__ s_w, int64_t M,
                                                              int64_t O, int64_t Kb, uint16_t* __restrict__ Y, int64_t ldy, void* __restrict__ ws)
{
    typedef Mma<DT> MM;
    typedef typename MM::dfrag_t frag_t;
    constexpr int SUB = MM::DENSE_SUB, NSUB = 128 / SUB, RPF = SUB / 32;   // k-bytes per instruction, instructions per unit, 16-byte pieces per fragment
    __shared__ __attribute__((aligned(16))) uint8_t red[(SK_WAVES - 1) * FPW * TB * 16 * 64 * 4];
    __shared__ __attribute__((aligned(128))) uint8_t tile[SK_WAVES][FPW * 32 * 128];   // per wavefront: FPW x 32 weight rows x 128 bytes
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t o0 = (int64_t)blockIdx.x * (32 * FPW);
    const int U = (int)(Kb / 128);
    // weight lines: load j (0..3) of fragment f covers row 32 f + 8 j + lane / 8, 16-byte chunk lane % 8 of the unit
    const uint8_t* wp[FPW][4];
    int wofs[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 8 * j + (lane >> 3), chunk = lane & 7;
        wofs[j] = row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);            // 16-byte XOR swizzle against bank conflicts
#pragma unroll
        for (int f = 0; f < FPW; ++f) {
            int64_t o = o0 + 32 * f + row;
            o = o < O ? o : O - 1;
            wp[f][j] = Wq + o * Kb + 16 * chunk;
        }
    }
    // fragment reads: lane (i, q) reads row sk_frag_row(i)
    const int frow = sk_frag_row(lane & 31), q = lane >> 5;
    // token rows: lane (n, q) holds bytes [q SUB / 2, (q + 1) SUB / 2) of token n within an instruction's k range
    const uint8_t* xb[TB];
    bool live[TB];                                       // lanes without a token load nothing (see the sparse kernel)
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        int64_t tok = tb * 32 + (lane & 31);
        live[tb] = tok < M;
        tok = live[tb] ? tok : M - 1;
        xb[tb] = Xq + tok * Kb + (SUB / 2) * q;
    }
    auto load = [&](SkDenseUnit<TB, FPW>& R, int u) {
#pragma unroll
        for (int f = 0; f < FPW; ++f)
#pragma unroll
            for (int j = 0; j < 4; ++j) R.a[f][j] = *reinterpret_cast<const v4i*>(wp[f][j] + (int64_t)u * 128);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
            if (live[tb]) {
#pragma unroll
                for (int t = 0; t < NSUB; ++t)
#pragma unroll
                    for (int piece = 0; piece < RPF; ++piece)
                        R.b[tb][t * RPF + piece] = *reinterpret_cast<const v4i*>(xb[tb] + (int64_t)u * 128 + t * SUB + 16 * piece);
            }
    };
    typename MM::acc_t acc[FPW * TB];
#pragma unroll
    for (int i = 0; i < FPW * TB; ++i) sk_zero(acc[i]);
    constexpr int D = SK_DEPTH<FPW, TB>;                     // register stages in flight per wavefront (see the sparse kernel)
    SkDenseUnit<TB, FPW> st[D];
#pragma unroll
    for (int d = 0; d < D; ++d)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int j = 0; j < 4; ++j) st[d].b[tb][j] = v4i{0, 0, 0, 0};
    uint8_t* my = tile[wave];
    const int u_end = (int)((int64_t)(blockIdx.y + 1) * U / gridDim.y);
    const int u0 = (int)((int64_t)blockIdx.y * U / gridDim.y) + wave;
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (u0 + d * SK_WAVES < u_end) load(st[d], u0 + d * SK_WAVES);
    for (int ub = u0; ub < u_end; ub += D * SK_WAVES) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const int u = ub + d * SK_WAVES;
        if (u >= u_end) continue;
        SkDenseUnit<TB, FPW>& cur = st[d];
        // lines -> wavefront-private LDS tile -> fragments (LDS operations of one wavefront execute in order)
#pragma unroll
        for (int f = 0; f < FPW; ++f)
#pragma unroll
            for (int j = 0; j < 4; ++j) *reinterpret_cast<v4i*>(my + f * 4096 + wofs[j]) = cur.a[f][j];
#pragma unroll
        for (int t = 0; t < NSUB; ++t) {
            frag_t b[TB];
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int piece = 0; piece < RPF; ++piece)
#pragma unroll
                    for (int e = 0; e < 4; ++e) b[tb][4 * piece + e] = cur.b[tb][t * RPF + piece][e];
#pragma unroll
            for (int f = 0; f < FPW; ++f) {
                frag_t a;
#pragma unroll
                for (int piece = 0; piece < RPF; ++piece) {
                    const int lc = t * (SUB / 16) + q * RPF + piece;
                    const v4i v = *reinterpret_cast<const v4i*>(my + f * 4096 + frow * 128 + ((lc ^ ((frow >> 1) & 7)) << 4));
#pragma unroll
                    for (int e = 0; e < 4; ++e) a[4 * piece + e] = v[e];
                }
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) acc[f * TB + tb] = MM::dense(a, b[tb], acc[f * TB + tb]);
            }
        }
        if (u + D * SK_WAVES < u_end) load(cur, u + D * SK_WAVES);
      }
    }
    sk_reduce<SK_WAVES, typename MM::acc_t, FPW * TB>(acc, red, wave, lane);
    if (wave == 0) {
        if (gridDim.y > 1) { sk_store_partial<typename MM::acc_t, FPW * TB>(acc, ws, (int)blockIdx.x, lane); return; }
#pragma unroll
        for (int f = 0; f < FPW; ++f) {
            typename MM::acc_t part[TB];
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) part[tb] = acc[f * TB + tb];
            sk_store<MM::SCALED, typename MM::acc_t, TB>(part, s_x, s_w, Y, ldy, M, O, o0 + 32 * f + 16 * (lane >> 5), lane);
        }
    }
}

// Split k: sum of the S partial accumulators of fragment blockIdx.x in range order and the scale epilogue.  Thread
// (tb, register quad r4, lane) owns four consecutive channels of one token, so a range costs it one 16-byte load and
// the loads of up to eight ranges are in flight at once: the kernel is one or two memory round trips long.
// PANEL_ORDER: fragment F is fragment F % 4 of weight panel F / 4 (channels panel * 128 + 64 h + 16 (F % 4) + r);
// otherwise it is channels 32 F + 16 h + r.
template <int DT, int TB, bool PANEL_ORDER>
__global__ __launch_bounds__(256 * TB) void k_skinny_reduce(const v4i* __restrict__ ws, int S, const float* __restrict__ s_x,
                                                           const float* __restrict__ s_w, int64_t M, int64_t O, uint16_t* __restrict__ Y, int64_t ldy)
{
    typedef Mma<DT> MM;
    typedef typename MM::acc_t acc_t;
    typedef decltype(acc_t{}[0] + acc_t{}[0]) elem_t;
    typedef elem_t quad_t __attribute__((ext_vector_type(4)));
    const int64_t F = blockIdx.x, nfrag = gridDim.x;
    const int lane = threadIdx.x & 63, r4 = (threadIdx.x >> 6) & 3, tb = threadIdx.x >> 8, h = lane >> 5;
    quad_t a = {0, 0, 0, 0};
    const v4i* src = ws + ((F * TB + tb) * 4 + r4) * 64 + lane;
    const int64_t range_stride = nfrag * TB * 4 * 64;
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
    const int64_t o = (PANEL_ORDER ? (F >> 2) * PANEL + 64 * h + 16 * (F & 3) : F * 32 + 16 * h) + 4 * r4;
    store_quad4<MM::SCALED>(a, s_x, s_w, Y, ldy, M, O, o, tb * 32 + (lane & 31));
}

}  // namespace ss

using namespace ss;

// Fragments per workgroup: as many (4, 2 or 1) as leave every compute unit at least one workgroup.
static int pick_fpw(int64_t frags)
{
    const int cus = cu_count();
    int fpw = 4;
    while (fpw > 1 && frags / fpw < cus) fpw >>= 1;
    return fpw;
}

// U units of 128 bytes per token row (lifted rows, or unlifted rows when FUSED), ldxb bytes between rows
template <int DT, int TB, int FPW, bool FUSED>
static ss_status launch_sparse_one(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                                   int U, int64_t ldxb, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream)
{
    const int64_t npanels = (O + PANEL - 1) / PANEL;
    const unsigned grid = (unsigned)(npanels * (FRAGS_PER_PANEL / FPW));
    if (FPW == 1 && (int)grid < cu_count()) {
        hipLaunchKernelGGL((k_sparse_skinny<DT, TB, 1, 8, FUSED>), dim3(grid, (unsigned)S), dim3(512), 0, stream, static_cast<const uint8_t*>(XL), s_x,
                           static_cast<const uint8_t*>(w_vals), static_cast<const uint8_t*>(w_meta), s_w, M, O, U, ldxb, static_cast<uint16_t*>(Y), ldy, ws);
        const ss_status first = launch_status();       // reading the status clears it: keep it
        if (first != SS_OK || S <= 1) return first;
        hipLaunchKernelGGL((k_skinny_reduce<DT, TB, true>), dim3(grid), dim3(256 * TB), 0, stream, static_cast<const v4i*>(ws), S, s_x, s_w, M, O,
                           static_cast<uint16_t*>(Y), ldy);
    } else {
        // several fragments per workgroup; with S > 1 the k range is split over S workgroups per fragment group
        hipLaunchKernelGGL((k_sparse_skinny<DT, TB, FPW, 4, FUSED>), dim3(grid, (unsigned)S), dim3(256), 0, stream, static_cast<const uint8_t*>(XL), s_x,
                           static_cast<const uint8_t*>(w_vals), static_cast<const uint8_t*>(w_meta), s_w, M, O, U, ldxb, static_cast<uint16_t*>(Y), ldy, ws);
        const ss_status first = launch_status();
        if (first != SS_OK || S <= 1) return first;
        hipLaunchKernelGGL((k_skinny_reduce<DT, TB, true>), dim3((unsigned)(npanels * FRAGS_PER_PANEL)), dim3(256 * TB), 0, stream,
                           static_cast<const v4i*>(ws), S, s_x, s_w, M, O, static_cast<uint16_t*>(Y), ldy);
    }
    return launch_status();
}

template <int DT, int TB, int FPW>
static ss_status launch_dense_one(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, void* Y,
                                  int64_t ldy, void* ws, int S, hipStream_t stream)
{
    const unsigned grid = (unsigned)((O + 32 * FPW - 1) / (32 * FPW));
    if (FPW == 1 && (int)grid < cu_count()) {
        hipLaunchKernelGGL((k_dense_skinny<DT, TB, 1, 8>), dim3(grid, (unsigned)S), dim3(512), 0, stream, static_cast<const uint8_t*>(Xq), s_x,
                           static_cast<const uint8_t*>(Wq), s_w, M, O, Kb, static_cast<uint16_t*>(Y), ldy, ws);
        const ss_status first = launch_status();
        if (first != SS_OK || S <= 1) return first;
        hipLaunchKernelGGL((k_skinny_reduce<DT, TB, false>), dim3(grid), dim3(256 * TB), 0, stream, static_cast<const v4i*>(ws), S, s_x, s_w, M, O,
                           static_cast<uint16_t*>(Y), ldy);
    } else
        hipLaunchKernelGGL((k_dense_skinny<DT, TB, FPW, 4>), dim3(grid), dim3(256), 0, stream, static_cast<const uint8_t*>(Xq), s_x,
                           static_cast<const uint8_t*>(Wq), s_w, M, O, Kb, static_cast<uint16_t*>(Y), ldy, ws);
    return launch_status();
}

// k ranges when workgroups are single 32-channel fragments (fewer fragments, counted in whole panels, than compute
// units; eight wavefronts each): every wavefront keeps at least eight units, at most `cap` ranges.  Measured on
// 18944 -> 3584 (112 fragments, INT8 6:8): M = 16 28 -> 20 us, M = 32 37 -> 24 us; at M = 1 the second kernel costs
// what the split saves, so fewer than 8 tokens are not split.
static int frag_splits(int64_t M, int64_t O, int64_t units, int cap)
{
    const int64_t nfrag = (O + PANEL - 1) / PANEL * FRAGS_PER_PANEL;
    const int cus = cu_count();
    if (M < 8 || nfrag >= cus) return 1;
    int64_t S = cus / nfrag;
    if (S > units / 64) S = units / 64;
    if (S > cap) S = cap;
    return S < 2 ? 1 : (int)S;
}

// k ranges when workgroups are whole 128-channel panels (sparse kernel, rows of at least 64 units on fewer panels than
// compute units): one workgroup per compute unit, ranges of at least 32 units.  Measured on 18944 -> 3584 (28 panels,
// INT8 6:8; single fragments unsplit -> panels in 4..7 ranges): M = 1 19 -> 16 us, M = 16 28 -> 17 us, M = 32 37 -> 19 us;
// on rows of 42 units (3584 -> 4608) the second kernel costs more than the split saves.
static int panel_splits(int64_t O, int64_t units, int cap)
{
    const int64_t npanels = (O + PANEL - 1) / PANEL;
    const int cus = cu_count();
    if (npanels >= cus) return 1;
    int64_t S = cus / npanels;
    if (S > units / 32) S = units / 32;
    if (S > cap) S = cap;
    return S < 2 ? 1 : (int)S;
}

// token blocks of 32: 1 (M <= 32) or 2 (M <= 64).  S = the ranges the workspace has room for.
template <int DT, bool FUSED>
static ss_status launch_sparse_dt(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                                  int U, int64_t ldxb, void* Y, int64_t ldy, void* ws, int S, hipStream_t st)
{
    const int64_t frags = (O + PANEL - 1) / PANEL * FRAGS_PER_PANEL;
    int fpw = pick_fpw(frags);
    // Long rows on few panels: whole panels per workgroup (the token rows are read once per 128 channels instead of once
    // per 32) with the k range split over enough workgroups to fill the chip; otherwise S only applies to single fragments.
    const int s4 = panel_splits(O, U, S);
    int s_use = fpw == 1 ? frag_splits(M, O, U, S) : 1;
    if (s4 > 1) { fpw = 4; s_use = s4; }
#define SS_GO(TB, FPW) return launch_sparse_one<DT, TB, FPW, FUSED>(XL, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, s_use, st)
    if (M <= 32) { if (fpw == 4) SS_GO(1, 4); if (fpw == 2) SS_GO(1, 2); SS_GO(1, 1); }
    if (fpw == 4) SS_GO(2, 4);
    if (fpw == 2) SS_GO(2, 2);
    SS_GO(2, 1);
#undef SS_GO
}

template <int DT>
static ss_status launch_dense_dt(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, void* Y,
                                 int64_t ldy, void* ws, int S, hipStream_t st)
{
    // One fragment per workgroup: the dense kernel stages its weight lines through LDS, and more fragments per
    // workgroup cost more in occupancy than they save in token re-reads (measured: 21 vs 35 us on 3584 -> 37888).
    const int s_use = frag_splits(M, O, Kb / KSTEP, S);
    if (M <= 32) return launch_dense_one<DT, 1, 1>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, s_use, st);
    return launch_dense_one<DT, 2, 1>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, s_use, st);
}

// Host side, called by the C entry points for M <= SS_SKINNY_MAX_M.  Arguments are already validated.
namespace ss {

// Number of k ranges the few-token kernels may use with a workspace of ws_bytes: the larger of what the two split
// policies above would take (the launchers apply their own policy below this bound).
int skinny_splits(int64_t M, int64_t O, int64_t units, size_t ws_bytes)
{
    if (M > SS_SKINNY_MAX_M) return 1;
    const size_t per_range = skinny_workspace_bytes(M, O, 2) / 2;
    const int64_t fit = (int64_t)(ws_bytes / per_range);
    const int cap = fit > 64 ? 64 : (int)fit;
    const int a = frag_splits(M, O, units, cap), b = panel_splits(O, units, cap);
    return a > b ? a : b;
}

size_t skinny_workspace_bytes(int64_t M, int64_t O, int S)
{
    const int64_t nfrag = (O + PANEL - 1) / PANEL * FRAGS_PER_PANEL;
    const int tb = M <= 32 ? 1 : 2;
    return S > 1 ? (size_t)S * nfrag * tb * 16 * 64 * 4 : 0;
}

ss_status launch_sparse_skinny(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                               int64_t Kpb, ss_dtype dtype, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream)
{
    const int U = (int)(Kpb / KSTEP);
    switch (dtype) {
    case SS_I8: return launch_sparse_dt<SS_I8, false>(XL, s_x, w_vals, w_meta, s_w, M, O, U, Kpb, Y, ldy, ws, S, stream);
    case SS_FP8_E4M3: return launch_sparse_dt<SS_FP8_E4M3, false>(XL, s_x, w_vals, w_meta, s_w, M, O, U, Kpb, Y, ldy, ws, S, stream);
    case SS_BF16: return launch_sparse_dt<SS_BF16, false>(XL, s_x, w_vals, w_meta, s_w, M, O, U, Kpb, Y, ldy, ws, S, stream);
    case SS_FP16: return launch_sparse_dt<SS_FP16, false>(XL, s_x, w_vals, w_meta, s_w, M, O, U, Kpb, Y, ldy, ws, S, stream);
    }
    return SS_ERR_DTYPE;
}

ss_status launch_sparse_fused_skinny(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                                     int U, int64_t ldxb, ss_dtype dtype, void* Y, int64_t ldy, void* ws, int S, hipStream_t stream)
{
    switch (dtype) {
    case SS_I8: return launch_sparse_dt<SS_I8, true>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, stream);
    case SS_FP8_E4M3: return launch_sparse_dt<SS_FP8_E4M3, true>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, stream);
    case SS_BF16: return launch_sparse_dt<SS_BF16, true>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, stream);
    case SS_FP16: return launch_sparse_dt<SS_FP16, true>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, ws, S, stream);
    }
    return SS_ERR_DTYPE;
}

ss_status launch_dense_skinny(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, ss_dtype dtype,
                              void* Y, int64_t ldy, void* ws, int S, hipStream_t stream)
{
    switch (dtype) {
    case SS_I8: return launch_dense_dt<SS_I8>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, stream);
    case SS_FP8_E4M3: return launch_dense_dt<SS_FP8_E4M3>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, stream);
    case SS_BF16: return launch_dense_dt<SS_BF16>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, stream);
    case SS_FP16: return launch_dense_dt<SS_FP16>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, ws, S, stream);
    }
    return SS_ERR_DTYPE;
}

}  // namespace ss
