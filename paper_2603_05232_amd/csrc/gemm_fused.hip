// slide_sparse_gemm_fused: the 2:4 sparse GEMM of the 6:8 pattern (N = 4) on UNLIFTED quantised activations.
// The lifting operator (Sec. 3.3; window j = g(N-1)+l of a row starts at b = 2N g + 2l, Alg. 1) is applied on the way
// from LDS to the operand registers, so the lifted matrix X' (1.5 K bytes per token) is never written, read or staged:
// token tiles move K bytes per token from L2 to LDS and from LDS to registers.
//
// K loop.  A super-unit is 128 unlifted bytes of a token row (one cache line) = 16 blocks of 8 bytes = 48 windows
// = three sparse matrix instructions deep (64 lifted bytes each).  B lane (n, qb) reads its 64 bytes of the line as
// 16 registers; the first eight are the B operand of step 0 as they are (windows l = 0 and l = 2 of four blocks are
// the blocks' two halves), the second eight of step 1, and step 2 takes the eight middle windows (l = 1), each built
// with one v_alignbyte (8-bit types) or two register copies (16-bit types).  slide_decompose_fused packs the weights
// in the matching window order (fused_window in packed_layout.h).
//
// Tile engine.  Persistent workgroups, 256 channels x 256 tokens per tile, 2 x WT wavefronts of 128 channels x
// (256 / WT) tokens = 4 x NBF accumulator blocks of the 32x32 instruction.  WT = 4 (eight wavefronts, two per SIMD) is
// what is built: with WT = 2 (four wavefronts of 128 x 128, a third fewer LDS operand reads) a lone wavefront could not
// keep its SIMD's matrix pipe busy and the kernel was 7-10 % slower.  Operands go L2 -> LDS with direct loads into
// two rings: token tiles (32 KB per super-unit, three slots) and packed weights (10 KB per step: 8 KB of stored values
// + 2 KB of index words, six slots).  The workgroup meets at one barrier per super-unit; a wavefront issues all LDS
// reads of a step's operands at least one step ahead and the reads of the step before a barrier in that step's first
// half, so no wait is exposed; the direct loads of later super-units are spread one by one between the matrix
// instructions.  The next tile's first operands are requested before the epilogue and waited for inside it, before
// the first store: the wait counter counts stores too, and a wait behind them would wait for their acknowledgement.
//
// Token tile in LDS: 256 rows x 128 bytes, the 16-byte chunk c of row r stored at chunk c ^ ((r >> 1) & 7) (the
// swizzle is applied on the global-address side: a direct load writes 64 lanes x 16 bytes contiguously, i.e. eight
// whole rows, and the eight lanes of a row fetch its cache line in permuted order).  For a fixed chunk the sixteen
// lanes of an LDS read phase (sixteen consecutive rows) land on sixteen different 16-byte bank groups; a B lane
// keeps the four addresses of its chunks 4 qb .. 4 qb + 3.
#include "ss_common.h"
#include "packed_layout.h"
#include "mma_types.h"
#include "lds_pipe.h"
#include "tile_common.h"
#include "device_info.h"
#include <type_traits>

namespace ss {

constexpr int F_ASTEP = 10 * 1024;                    // one step of both panels: values [panel 2][fragment 4][lane 64][16 B], index words [panel 2][lane 64][fragment 4][4 B]
constexpr int F_AIDX = 8 * 1024;                      // offset of the index words inside a step slot
constexpr int F_ARING = 6;
constexpr int F_BSLOT = 32 * 1024;
constexpr int F_BRING = 3;
constexpr int F_B_OFF = F_ARING * F_ASTEP;            // 60 KB
constexpr int F_SW_OFF = F_B_OFF + F_BRING * F_BSLOT; // 156 KB
constexpr int F_SWB = BO * 4;                         // the tile's channel scales; two copies (this tile, next tile)
constexpr int F_LDS = F_SW_OFF + 2 * F_SWB;           // 158 KB
static_assert(F_LDS <= 160 * 1024, "LDS budget");

// wait until at most N of this wavefront's loads are in flight; LDS reads are left alone
template <int N> __device__ inline void wait_vm_only()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
    asm volatile("" ::: "memory");
}

enum { IT_STEADY = 0, IT_TAIL = 1, IT_LAST = 2 };

template <int DT, int WT>
__global__ __launch_bounds__(128 * WT) void k_sparse_fused(const uint8_t* __restrict__ Xq, const float* __restrict__ s_x, const uint8_t* __restrict__ w_vals,
                                                            const uint8_t* __restrict__ w_meta, const float* __restrict__ s_w, int64_t M, int64_t O, int U,
                                                            int64_t ldxb, uint16_t* __restrict__ Y, int64_t ldy, int tiles_o, int tiles_t)
{
    typedef Mma<DT> MM;
    constexpr int W = 2 * WT, NBF = 8 / WT, NM = 4 * NBF, ES = MM::ES;
    constexpr int LB = 32 / W;                       // token-tile loads per wavefront and super-unit (1 KB each)
    constexpr int APS = 8 / W;                       // 1 KB pieces of stored values per wavefront and step
    constexpr int IPW = (6 + W - 1) / W;             // 1 KB pieces of index words per wavefront and super-unit (6 per tile: 2 panels x 3 steps; spare turns repeat a piece)
    constexpr int LG = 3 * APS + IPW;                // weight loads per wavefront and super-unit
    constexpr int L = LG + LB;
    constexpr int EP_ROWS = 128 / W;                 // rows per wavefront staged at a time: W x EP_ROWS x 256 B = 32 KB, one ring slot
    static_assert(L <= (3 * NM) / 2, "one direct load behind every second matrix instruction");
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wo = wave & 1, wt = wave >> 1;
    const int n = lane & 31, qb = lane >> 5;
    const uint32_t lds0 = lds_address(smem);
    const int nsteps = 3 * U;
    const int64_t npanels = (O + PANEL - 1) / PANEL;
    const int pw = (wave * APS) >> 2, f0 = (wave * APS) & 3;            // this wavefront's weight pieces: panel pw of the tile, fragments f0 .. f0 + APS - 1
    const uint32_t a_wave = lds0 + pw * 4096 + f0 * 1024;
    int ip[IPW], ij[IPW];                           // this wavefront's index-word pieces in the steady state: panel, step within the super-unit
#pragma unroll
    for (int e = 0; e < IPW; ++e) { const int q = (wave + e * W) % 6; ip[e] = q / 3; ij[e] = q % 3; }
    const uint32_t b_wave = lds0 + F_B_OFF + wave * 1024;
    const uint32_t lane16 = lane * 16;

    // LDS byte offsets of this lane's operand reads (ring slot and fragment / chunk are added as they come)
    const uint32_t va = wo * 4096 + lane * 16, vi = F_AIDX + wo * 1024 + lane * 16;
    uint32_t vb[NBF][4];                             // per token fragment: the lane's four chunks of a line
#pragma unroll
    for (int bb = 0; bb < NBF; ++bb) {
        const int R = wt * (32 * NBF) + 32 * bb + n;
#pragma unroll
        for (int j = 0; j < 4; ++j) vb[bb][j] = F_B_OFF + R * ROWB + 16 * ((4 * qb + j) ^ swz(R));
    }

    // Per-tile state of the loaders, set up for the next tile before the current tile's epilogue.
    const uint8_t *b_src = nullptr, *av_src = nullptr, *am_tile[2] = {nullptr, nullptr};
    uint32_t boff[LB];
    int64_t o_blk = 0, t_blk = 0;
    auto setup_tile = [&](int to, int tt) {
        o_blk = (int64_t)to * BO;
        t_blk = (int64_t)tt * BT;
        const int ln = fresh_lane();
        b_src = Xq + t_blk * ldxb;
        const int64_t left = M - t_blk;               // >= 1
        const int last = left > 255 ? 255 : (int)left - 1;
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int row = 8 * (i * W + wave) + (ln >> 3);
            boff[i] = (uint32_t)(row < last ? row : last) * (uint32_t)ldxb + ((ln & 7) ^ swz(row)) * 16;
        }
        int64_t panel = (int64_t)to * 2 + pw;
        panel = panel < npanels ? panel : npanels - 1;
        av_src = w_vals + (panel * nsteps * 4 + f0) * 1024;
#pragma unroll
        for (int pp = 0; pp < 2; ++pp) {
            int64_t pn = (int64_t)to * 2 + pp;
            pn = pn < npanels ? pn : npanels - 1;
            am_tile[pp] = w_meta + pn * nsteps * 1024;
        }
    };
    // the weight loads of step k into ring slot `aslot` (the index words of the two panels by wavefronts 0 and 1), the
    // LB token loads of super-unit u into ring slot `bslot`
    auto load_a_step = [&](int k, int aslot) {
        const uint8_t* av = av_src + (int64_t)k * 4096;
#pragma unroll
        for (int e = 0; e < APS; ++e) lds_dma16_at(av + e * 1024, lane16, a_wave + aslot * F_ASTEP + e * 1024);
        if (wave < 2) lds_dma16_at((wave ? am_tile[1] : am_tile[0]) + (int64_t)k * 1024, lane16, lds0 + aslot * F_ASTEP + F_AIDX + wave * 1024);
    };
    auto load_b_unit = [&](int u, int bslot) {
#pragma unroll
        for (int i = 0; i < LB; ++i) lds_dma16_at(b_src + (int64_t)u * 128, boff[i], b_wave + bslot * F_BSLOT + i * W * 1024);
    };
    auto load_scales = [&](int parity) {
        if constexpr (MM::SCALED) {
            const int64_t o_first = o_blk + (wave & 3) * 64, left = O - 1 - o_first;     // clamp to the last channel
            const int left32 = left > 63 ? 63 : (int)left, ln = fresh_lane();
            const uint32_t oc = left32 < 0 ? 0u : (uint32_t)(ln < left32 ? ln : left32);
            lds_dma4_at(reinterpret_cast<const uint8_t*>(s_w + (left < 0 ? O - 1 : o_first)), oc * 4, lds0 + F_SW_OFF + parity * F_SWB + (wave & 3) * 256);
        }
    };
    // loads requested before the epilogue of the previous tile: step 0, token tile 0, steps 1..3, scales, (token tile 1)
    auto request_head = [&](int parity) {
        load_a_step(0, 0);
        load_b_unit(0, 0);
#pragma unroll
        for (int k = 1; k <= 3; ++k) if (k < nsteps) load_a_step(k, k);
        load_scales(parity);
        if (U > 1) load_b_unit(1, 1);
    };
    uint8_t* const stage = smem + F_B_OFF + 2 * F_BSLOT + wave * (EP_ROWS * EP_ROWB);

    struct Regs { v4i aA[4], a[4], iA, iB, iC; v8i lo[NBF], hi[NBF], al[NBF]; };

    int to, tt;
    bool have = tile_of_round(0, tiles_o, tiles_t, to, tt);
    if (have) { setup_tile(to, tt); request_head(0); }
    for (int round = 0; have; ++round) {
        typename MM::acc_t acc[4][NBF];
        zero_acc(acc);
        Regs R;
        auto rd = [&](uint32_t off) -> v4i { return *reinterpret_cast<const v4i*>(smem + off); };
        auto mma = [&](typename MM::acc_t& c, v4i a, const v8i& b, int idx) __attribute__((always_inline)) { c = MM::sparse(a, b, c, idx); };
        // the four 16-byte reads of token fragment bb's half `hi` (chunks 2 hi, 2 hi + 1 of the lane's 64 bytes)
        auto read_b = [&](v8i& dst, const uint32_t (&vbs)[4], int half, int piece) {
            const v4i v = rd(vbs[2 * half + piece]);
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[4 * piece + e] = v[e];
        };
        // middle windows of fragment b's blocks: al[jd], 8-bit: bytes 2..5 of block jd; 16-bit: elements 2..5 of block jd >> 1, half jd & 1
        auto make_al = [&](int b, int jd) {
            if constexpr (ES == 1) {
                const int lo_i = 2 * jd;              // registers 2 jd, 2 jd + 1 of the lane's 16
                const uint32_t x0 = lo_i < 8 ? (uint32_t)R.lo[b][lo_i & 7] : (uint32_t)R.hi[b][lo_i & 7];
                const uint32_t x1 = lo_i < 8 ? (uint32_t)R.lo[b][(lo_i + 1) & 7] : (uint32_t)R.hi[b][(lo_i + 1) & 7];
                R.al[b][jd] = (int)__builtin_amdgcn_alignbyte(x1, x0, 2);
            } else {
                const int src = 4 * (jd >> 1) + 1 + (jd & 1);
                R.al[b][jd] = src < 8 ? R.lo[b][src] : R.hi[b][src - 8];
            }
        };

        // One super-unit u.  `par` = (u & 1) * 3 is the ring slot of its first step; `bn` the ring slot of token tile
        // u + 1 (read during this super-unit), so tile u + 3 goes where tile u was.  IT_STEADY: the L direct loads of
        // steps 3u+4 .. 3u+6 and of token tile u+3 go one by one behind every second matrix instruction; IT_TAIL:
        // whatever is left of the weights is requested up front; IT_LAST: nothing follows this super-unit.
        auto super_unit = [&](auto mode_c, int u, int par, int bn) __attribute__((always_inline)) {
            constexpr int MODE = decltype(mode_c)::value;
            constexpr bool NEXT = MODE != IT_LAST;
            // the first matrix instruction goes out right behind the barrier; the scalar set-up of this super-unit's
            // direct loads (below) runs in its shadow instead of ahead of it
            __builtin_amdgcn_sched_barrier(0);
            mma(acc[0][0], R.aA[0], R.lo[0], R.iA[0]);
            __builtin_amdgcn_sched_barrier(0);
            const uint32_t a_now = va + par * F_ASTEP, i_now = vi + par * F_ASTEP;               // steps 3u .. 3u+2
            const uint32_t a_nxt = va + (3 - par) * F_ASTEP, i_nxt = vi + (3 - par) * F_ASTEP;     // step 3u+3
            uint32_t vbn[NBF][4];
#pragma unroll
            for (int bb = 0; bb < NBF; ++bb)
#pragma unroll
                for (int j = 0; j < 4; ++j) vbn[bb][j] = vb[bb][j] + bn * F_BSLOT;
            // scalar parts of the direct loads of this iteration: steps k_ld .. k_ld + 2 go to ring slots par + 4, par + 5, par (mod 6)
            const int k_ld = 3 * u + 4;
            const uint8_t* av = av_src + (int64_t)k_ld * 4096;
            const uint32_t s4 = (par == 0 ? 4 : 1) * F_ASTEP, s5 = (par == 0 ? 5 : 2) * F_ASTEP, s6 = (par == 0 ? 0 : 3) * F_ASTEP;
            const uint8_t* am[IPW];
            uint32_t im[IPW];                         // this wavefront's index-word pieces: source, LDS destination
#pragma unroll
            for (int e = 0; e < IPW; ++e) {
                am[e] = (ip[e] ? am_tile[1] : am_tile[0]) + (int64_t)(k_ld + ij[e]) * 1024;
                im[e] = lds0 + F_AIDX + ip[e] * 1024 + (ij[e] == 0 ? s4 : ij[e] == 1 ? s5 : s6);
            }
            const uint8_t* bsrc = b_src + (int64_t)(u + 3) * 128;
            const uint32_t b_ld = b_wave + (bn == 0 ? 2 : bn - 1) * F_BSLOT;
            if constexpr (MODE == IT_TAIL) {
                if (k_ld < nsteps) load_a_step(k_ld, par == 0 ? 4 : 1);
                if (k_ld + 1 < nsteps) load_a_step(k_ld + 1, par == 0 ? 5 : 2);
                if (k_ld + 2 < nsteps) load_a_step(k_ld + 2, par == 0 ? 0 : 3);
            }
            // behind matrix instruction gi (0 .. 3 NM - 1) of the super-unit: direct load number gi / 2 if gi is odd
            auto after = [&](int gi) __attribute__((always_inline)) {
                if constexpr (MODE == IT_STEADY) {
                    const int d = gi >> 1;
                    if ((gi & 1) && d < L) {
                        if (d < 3 * APS) {
                            const int jj = d / APS, x = d % APS;
                            const uint32_t so = jj == 0 ? s4 : jj == 1 ? s5 : s6;
                            lds_dma16_at(av + jj * 4096 + x * 1024, lane16, a_wave + so + x * 1024);
                        } else if (d < LG) {
                            lds_dma16_at(am[d - 3 * APS], lane16, im[d - 3 * APS]);
                        } else {
                            const int i = d - LG;
                            lds_dma16_at(bsrc, boff[i < LB ? i : 0], b_ld + i * W * 1024);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            };
            // the operand reads that can go anywhere in a step are issued in its first slots: r-th read of a list of `cnt`
            // behind matrix instruction i when spread over the first `span` instructions
            auto mine = [](int r, int cnt, int span, int i) { return i < span && r >= (i * cnt) / span && r < ((i + 1) * cnt) / span; };

            // ---- step 0: registers 0..7 of the lane's line.  Reads the weights of step 1 (R.a is free: this step uses R.aA)
            // and builds the middle windows (second half: their last inputs were read during the previous step)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                if (i > 0) mma(acc[i / NBF][i % NBF], R.aA[i / NBF], R.lo[i % NBF], R.iA[i / NBF]);
                __builtin_amdgcn_sched_barrier(0);
                if (i < 4) R.a[i] = rd(a_now + F_ASTEP + i * 1024);
                if (i == 4) R.iB = rd(i_now + F_ASTEP);
                if (i >= NM / 2) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) { const int t = (i - NM / 2) * 4 + e; make_al(t / 8, t % 8); }
                }
                __builtin_amdgcn_sched_barrier(0);
                after(i);
            }
            // ---- step 1: registers 8..15.  The weights of step 2 refill R.a behind each fragment's last use; registers 0..7
            // are free and take the next line's first half
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                mma(acc[i / NBF][i % NBF], R.a[i / NBF], R.hi[i % NBF], R.iB[i / NBF]);
                __builtin_amdgcn_sched_barrier(0);
                if (i % NBF == NBF - 1) R.a[i / NBF] = rd(a_now + 2 * F_ASTEP + (i / NBF) * 1024);
                if (i == 0) R.iC = rd(i_now + 2 * F_ASTEP);
                if constexpr (NEXT) {
#pragma unroll
                    for (int r = 0; r < 2 * NBF; ++r)
                        if (mine(r, 2 * NBF, NM - 2, i)) read_b(R.lo[r >> 1], vbn[r >> 1], 0, r & 1);
                }
                __builtin_amdgcn_sched_barrier(0);
                after(NM + i);
            }
            // ---- step 2: the middle windows.  Everything read here (weights of the next super-unit's step 0 into R.aA, the
            // next line's second half into registers 8..15) is issued in the first half, so it has returned by the barrier
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                mma(acc[i / NBF][i % NBF], R.a[i / NBF], R.al[i % NBF], R.iC[i / NBF]);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (NEXT) {
#pragma unroll
                    for (int r = 0; r < 5 + 2 * NBF; ++r)
                        if (mine(r, 5 + 2 * NBF, NM / 2, i)) {
                            if (r < 4) R.aA[r] = rd(a_nxt + r * 1024);
                            else if (r == 4) R.iA = rd(i_nxt);
                            else read_b(R.hi[(r - 5) >> 1], vbn[(r - 5) >> 1], 1, (r - 5) & 1);
                        }
                }
                __builtin_amdgcn_sched_barrier(0);
                after(2 * NM + i);
            }
        };

        // ---- tile prologue: the head (requested before the previous epilogue) and the remaining token tiles
        // The head of this tile (requested before the previous epilogue) has landed: every wavefront waited for its
        // loads inside that epilogue, before its first store.  The first tile waits here.
        if (round == 0) wait_vm_only<0>();
        wg_barrier();                                 // head, scales and token tile 1 are published; the epilogue staging has been read out
#pragma unroll
        for (int f = 0; f < 4; ++f) R.aA[f] = rd(va + f * 1024);
        R.iA = rd(vi);
#pragma unroll
        for (int r = 0; r < 2 * NBF; ++r) { read_b(R.lo[r >> 1], vb[r >> 1], 0, r & 1); read_b(R.hi[r >> 1], vb[r >> 1], 1, r & 1); }
        // The first super-unit's direct loads go to the ring slots just read (step 0, token tile 0): every wavefront's
        // reads must have returned before any of those loads is issued.
        wait_lgkm0();
        wg_barrier();
        if (U > 2) load_b_unit(2, 2);                 // into the ring slot the staging used

        int u = 0, par = 0, bn = 1;
        for (; u + 3 < U; ++u) {
            super_unit(std::integral_constant<int, IT_STEADY>{}, u, par, bn);
            wait_vmcnt<LB>();                          // everything but the token tile just requested has landed; own reads have returned
            wg_barrier();
            par = 3 - par;
            bn = bn == 2 ? 0 : bn + 1;
        }
        for (; u + 1 < U; ++u) {
            super_unit(std::integral_constant<int, IT_TAIL>{}, u, par, bn);
            wait_vmcnt<0>();
            wg_barrier();
            par = 3 - par;
            bn = bn == 2 ? 0 : bn + 1;
        }
        // this sub-tile of Y and its token scales (requested here: they arrive behind the last matrix instructions)
        const int64_t o_sub = o_blk + wo * 128, t_sub = t_blk + wt * (32 * NBF);
        const int64_t rows = M - t_sub, cols = O - o_sub;          // <= 0: nothing of this sub-tile exists
        const bool any = rows > 0 && cols > 0;
        const int rows_left = any ? (int)(rows > 32 * NBF ? 32 * NBF : rows) : 0, cols_left = any ? (int)(cols > 128 ? 128 : cols) : 0;
        float sx[NBF];
        load_token_scales<MM::SCALED>(sx, MM::SCALED && any ? s_x + t_sub : s_x, rows_left);
        super_unit(std::integral_constant<int, IT_LAST>{}, u, par, bn);
        wg_barrier();                                 // every wavefront is done with the operand rings
        uint16_t* const Y_sub = any ? Y + t_sub * ldy + o_sub : Y;
        settle(sx);                                   // the token scales have arrived: no wait for them behind the loads requested next
        have = tile_of_round(round + 1, tiles_o, tiles_t, to, tt);
        if (have) { setup_tile(to, tt); request_head((round + 1) & 1); }
        store_tile<MM::SCALED, EP_ROWS, true>(acc, sx, reinterpret_cast<const float*>(smem + F_SW_OFF + (round & 1) * F_SWB) + wo * 128, Y_sub,
                                        (uint32_t)ldy, rows_left, cols_left, stage);
    }
}

}  // namespace ss

using namespace ss;

template <int DT, int WT>
static ss_status launch_fused(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O, int U,
                              int64_t ldxb, void* Y, int64_t ldy, hipStream_t stream)
{
    const int tiles_o = (int)((O + BO - 1) / BO), tiles_t = (int)((M + BT - 1) / BT);
    const int cus = cu_count(), ntiles = tiles_o * tiles_t;
    const int grid = ntiles < cus ? ntiles : cus;
    if (grid <= 0) return SS_ERR_HIP;
    if (allow_dynamic_lds<k_sparse_fused<DT, WT>>(F_LDS) != SS_OK) return SS_ERR_HIP;
    hipLaunchKernelGGL((k_sparse_fused<DT, WT>), dim3(grid), dim3(128 * WT), F_LDS, stream, static_cast<const uint8_t*>(Xq), s_x,
                       static_cast<const uint8_t*>(w_vals), static_cast<const uint8_t*>(w_meta), s_w, M, O, U, ldxb, static_cast<uint16_t*>(Y), ldy,
                       tiles_o, tiles_t);
    return launch_status();
}

static ss_status fused_gemm(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                            int64_t K, int64_t ldx, int N, ss_dtype dtype, void* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!valid_N(N) || N != 4) return SS_ERR_BAD_PATTERN_N;
    if (!valid_dtype(dtype)) return SS_ERR_DTYPE;
    const int es = elem_size(dtype);
    if (M < 0 || O < 0 || K <= 0 || (K * es) % KSTEP != 0 || ldx < K || (ldx * es) % 16 != 0 || ldy < O || M > (1 << 24) || ldy >= (1 << 22) ||
        ldx * es > (1 << 23))
        return SS_ERR_SHAPE;
    if (workspace_bytes > 0 && !workspace) return SS_ERR_NULL;
    if ((uintptr_t)workspace & 15) return SS_ERR_WORKSPACE;
    if (M == 0 || O == 0) return SS_OK;
    if (!Xq || !w_vals || !w_meta || !Y) return SS_ERR_NULL;
    if (!unscaled(dtype) && (!s_x || !s_w)) return SS_ERR_NULL;
    if (((uintptr_t)Xq & 15) || ((uintptr_t)w_vals & 15) || ((uintptr_t)w_meta & 15)) return SS_ERR_SHAPE;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int U = (int)(K * es / KSTEP);
    const int64_t ldxb = ldx * es;
    // kernel family by shape, as for the other two GEMMs; the k loop counts super-units of 128 unlifted bytes
    const ss_plan p = plan_gemm(M, O, U, workspace_bytes);
    if (p.path == SS_PATH_SKINNY) return launch_sparse_fused_skinny(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, dtype, Y, ldy, workspace, p.S, hs);
    if (p.path == SS_PATH_MID) return launch_sparse_fused_mid(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, dtype, Y, ldy, workspace, p.S, hs);
#define SS_F(DT) launch_fused<DT, 4>(Xq, s_x, w_vals, w_meta, s_w, M, O, U, ldxb, Y, ldy, hs)
    switch (dtype) {
    case SS_I8: return SS_F(SS_I8);
    case SS_FP8_E4M3: return SS_F(SS_FP8_E4M3);
    case SS_BF16: return SS_F(SS_BF16);
    case SS_FP16: return SS_F(SS_FP16);
    }
#undef SS_F
    return SS_ERR_DTYPE;
}

extern "C" ss_status slide_sparse_gemm_fused(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M,
                                             int64_t O, int64_t K, int64_t ldx, int N, ss_dtype dtype, void* Y, int64_t ldy, void* stream)
{
    return fused_gemm(Xq, s_x, w_vals, w_meta, s_w, M, O, K, ldx, N, dtype, Y, ldy, nullptr, 0, stream);
}

extern "C" ss_status slide_sparse_gemm_fused_ws(const void* Xq, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M,
                                                int64_t O, int64_t K, int64_t ldx, int N, ss_dtype dtype, void* Y, int64_t ldy, void* workspace,
                                                size_t workspace_bytes, void* stream)
{
    return fused_gemm(Xq, s_x, w_vals, w_meta, s_w, M, O, K, ldx, N, dtype, Y, ldy, workspace, workspace_bytes, stream);
}
