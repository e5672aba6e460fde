// Pieces shared by the 256 x 256 tile kernels (gemm.hip, gemm_fused.hip): the order in which persistent
// workgroups walk the output tiles, and the epilogue that stages a wavefront's accumulators through LDS so
// that every global store writes whole 256-byte row segments of Y.
#pragma once
#include "ss_common.h"
#include "mma_types.h"
#include "lds_pipe.h"

namespace ss {

constexpr int BO = 256;   // output channels per workgroup tile
constexpr int BT = 256;   // tokens per workgroup tile

// Persistent workgroups: the grid holds one workgroup per compute unit and workgroup b processes
// tiles b, b + grid, b + 2 grid, ...  Workgroup ids go round-robin to the 8 XCDs, so within a full
// round each XCD is given one contiguous run of tiles, and tiles are ordered in bands of 8 token
// tiles so that the 32 workgroups resident on an XCD share weight panels and token tiles in its L2.
__device__ inline bool tile_of_round(int round, int tiles_o, int tiles_t, int& to, int& tt)
{
    const int nb = gridDim.x, bid = blockIdx.x, total = tiles_o * tiles_t;
    const int base = round * nb;
    if (base + bid >= total) return false;
    int tile = base + bid;
    if (base + nb <= total && (nb & 7) == 0) tile = base + (bid & 7) * (nb >> 3) + (bid >> 3);
    constexpr int BAND = 8;
    const int per_band = BAND * tiles_o;
    const int band = tile / per_band, within = tile - band * per_band;
    const int bw = min(BAND, tiles_t - band * BAND);
    to = within / bw;
    tt = band * BAND + (within - to * bw);
    return true;
}

// ---- epilogue: Y = bf16((float(acc) * s_x) * s_w), staged through LDS for coalesced stores ------

// Staging holds ROWS (32 or 16) tokens x 128 channels of bf16 per wavefront at a time: rows of 256 bytes, ROWS / 4 KB
// per wavefront.  No row padding: the 16-byte chunk c of row r is stored at chunk c ^ (r & 15), which spreads both the
// column-wise writes and the row-wise reads over all banks.  With ROWS = 16 the 32 tokens of an accumulator column
// block go through in two passes (lanes of one half write, all lanes read and store), which halves the LDS the
// epilogue needs: kernels use it where that lets more of the next tile's operands be requested before the epilogue.
constexpr int EP_ROWB = 256;
constexpr int EP_WAVE_BYTES = 32 * EP_ROWB;         // 8 KB (ROWS = 32)

// token scales of this wavefront's sub-tile for the epilogue: sx[b] of lane (n, h) belongs to token 32 b + n.  Loaded
// ahead of the epilogue (callers issue this before the last k iterations) so that the latency is not exposed.
template <bool SCALED, int NB>
__device__ inline void load_token_scales(float (&sx)[NB], const float* __restrict__ s_x_sub, int rows_left)
{
    const int n = fresh_lane() & 31;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        sx[b] = 1.0f;
        if constexpr (SCALED) {
            uint32_t tk = (uint32_t)(b * 32 + n);
            tk = (int)tk < rows_left ? tk : (uint32_t)(rows_left - 1);
            if (rows_left > 0) sx[b] = s_x_sub[tk];
        }
    }
}

// Makes the compiler place its wait for the loads of sx here.  The kernels call it before they request the next tile's
// first operands with direct loads the compiler does not see: a wait placed behind those would count them in.
template <int NB> __device__ inline void settle(float (&sx)[NB])
{
#pragma unroll
    for (int b = 0; b < NB; ++b) asm volatile("" : "+v"(sx[b]));
}

// acc[f][b][r] of lane (n = lane & 31, h = lane >> 5) is channel 64 h + 16 f + r, token 32 b + n of this
// wavefront's 128-channel x (32 NB)-token sub-tile, whose first element is Y_sub (wave-uniform) and of which
// rows_left tokens x cols_left channels exist.  `stage` is this wavefront's private ROWS * 256 bytes of LDS;
// `sw_lds` holds the sub-tile's 128 channel scales in LDS (fetched with the tile's first unit), sx the token scales
// (load_token_scales).  All lane-dependent offsets are 32-bit (ldy < 2^22).
// SCALED = false (bf16 operands): Y = bf16(acc), the scales are not touched.
// SETTLE_LOADS: wait for every load this wavefront has in flight (the next tile's first operands, requested just before
// the epilogue) right before the first store is issued.  The wait counter counts loads and stores alike, so a later
// wait for those loads would also wait for the stores to be acknowledged; here the loads have had the first block's
// conversion to arrive and the stores are never waited for.
template <bool SCALED, int ROWS, bool SETTLE_LOADS, typename ACC, int NB>
__device__ inline void store_tile(const ACC (&acc)[4][NB], const float (&sx)[NB], const float* sw_lds, uint16_t* __restrict__ Y_sub,
                                  uint32_t ldy, int rows_left, int cols_left, uint8_t* stage)
{
    static_assert(ROWS == 32 || ROWS == 16, "staging rows");
    const int lane = fresh_lane(), n = lane & 31, h = lane >> 5;
    const bool vec_ok = ((ldy & 7) == 0) && (((uintptr_t)Y_sub & 15) == 0);
    const int seg = lane & 15;                      // 16-byte segment (8 channels) of the 256-byte row
    const int oc = 8 * seg;
    const uint32_t lane_elem = (uint32_t)(lane >> 4) * ldy + (uint32_t)oc;   // this lane's element offset in its first row
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        uint32_t w[4][8];
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            if constexpr (SCALED) {
                float sw[16];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float4 v = reinterpret_cast<const float4*>(sw_lds + 64 * h + 16 * f)[i];
                    sw[4 * i] = v.x; sw[4 * i + 1] = v.y; sw[4 * i + 2] = v.z; sw[4 * i + 3] = v.w;
                }
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    w[f][q] = pack_bf16x2(((float)acc[f][b][2 * q] * sx[b]) * sw[2 * q], ((float)acc[f][b][2 * q + 1] * sx[b]) * sw[2 * q + 1]);
            } else {
#pragma unroll
                for (int q = 0; q < 8; ++q) w[f][q] = pack_bf16x2((float)acc[f][b][2 * q], (float)acc[f][b][2 * q + 1]);
            }
        }
#pragma unroll
        for (int pass = 0; pass < 32 / ROWS; ++pass) {
            if (ROWS == 32 || (n >> 4) == pass) {
                uint8_t* row = stage + (n & (ROWS - 1)) * EP_ROWB;
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    const int c = h * 8 + 2 * f;    // first of the two 16-byte chunks of this lane's 16 channels
                    *reinterpret_cast<uint4*>(row + (((c) ^ (n & 15)) << 4)) = make_uint4(w[f][0], w[f][1], w[f][2], w[f][3]);
                    *reinterpret_cast<uint4*>(row + (((c + 1) ^ (n & 15)) << 4)) = make_uint4(w[f][4], w[f][5], w[f][6], w[f][7]);
                }
            }
            // wavefront-private staging: its own LDS writes only need to have completed
            if (SETTLE_LOADS && b == 0 && pass == 0) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < ROWS / 4; ++i) {
                const int r = 4 * i + (lane >> 4);
                const int tk = b * 32 + pass * ROWS + r;
                const uint4 v = *reinterpret_cast<const uint4*>(stage + r * EP_ROWB + ((seg ^ (r & 15)) << 4));
                if (tk < rows_left) {
                    uint16_t* dst = Y_sub + (lane_elem + (uint32_t)(b * 32 + pass * ROWS + 4 * i) * ldy);
                    if (vec_ok && oc + 8 <= cols_left) {
                        // Y is written once and not read again by this kernel: stream it past the caches
                        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                        __builtin_nontemporal_store((u32x4){v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4*>(dst));
                    } else {
                        const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (oc + e < cols_left) dst[e] = (uint16_t)(wv[e >> 1] >> (16 * (e & 1)));
                    }
                }
            }
            // the reads of this pass have returned (their data went out with the stores) before the next one is staged
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    }
}

template <typename ACC, int NB> __device__ inline void zero_acc(ACC (&acc)[4][NB])
{
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][b][r] = 0;
}

}  // namespace ss
