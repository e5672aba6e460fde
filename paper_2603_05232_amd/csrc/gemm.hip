// slide_sparse_gemm and dense_gemm for gfx950.
//
// Tile engine shared by both kernels: a persistent 512-thread workgroup (8 wavefronts, two per SIMD)
// owns a 256 (output channels) x 256 (tokens) tile of Y at a time; wavefront (wo, wt) accumulates the
// 128 x 64 sub-tile [wo*128, +128) x [wt*64, +64) as 4 x 2 blocks of a 32x32 matrix instruction.  The
// weights are the A operand (sparse for slide_sparse_gemm: the 32x32 sparse instructions take 16 bytes
// of stored values + one index word per lane), tokens are the B operand.  All k extents are counted in
// bytes of a row, so INT8, FP8 (e4m3) and BF16 share the kernels and differ in the matrix instruction,
// the accumulator type and the epilogue.
//
// Data movement.  Operand tiles go HBM/L2 -> LDS with direct-to-LDS loads (no registers hold data in
// flight) into rings of units; token rows are fetched as whole 128-byte lines and XOR-swizzled at
// 16-byte granularity (applied on the global-address side, because a direct load writes
// lane-contiguous LDS) so the 32 lanes of an operand read hit all 64 banks.
//
// Schedule.  The k loop advances in sub-steps of one matrix-instruction depth (64 lifted columns
// sparse, 32 columns dense): eight matrix instructions per wavefront, with the LDS reads of the next
// sub-step's operands (double-buffered registers) and a share of the direct loads of a later unit
// placed one by one between them -- a wavefront issues in order, and an LDS read or a load that has to
// wait for room in its queue keeps the matrix instructions behind it from issuing, so neither kind is
// issued in bursts.  The two wavefronts of a SIMD run freely against each other and fill each other's
// gaps; the workgroup meets at one barrier per unit (128 k-bytes), where the landed next unit is
// published and the ring slot of the finished unit is handed back to the loaders.
//
// Epilogue.  D[channel][token] leaves each lane with 64 consecutive output channels of one token; the
// scaled bf16 values are staged through LDS so that every global store instruction writes whole
// 256-byte row segments.  Staging takes 64 KB placed over ring slots the next tile's first unit does
// not use: that unit is requested before the epilogue and lands while the results are written out.
#include "ss_common.h"
#include "packed_layout.h"
#include "mma_types.h"
#include "lds_pipe.h"
#include "tile_common.h"
#include "device_info.h"
#include <atomic>
#include <type_traits>


namespace ss {

constexpr int G_WAVES = 8;
constexpr int G_THREADS = 64 * G_WAVES;
constexpr int NBF = 2;    // 32-token B fragments per wavefront (4 x 2 accumulator blocks of 32 x 32)

// ---- LDS tile of a row-major 8-bit operand: 256 rows x 128 bytes, XOR-swizzled -----------------

// per-thread source pointers (k offset 0) of the direct loads that fill a [256 x 128 B] tile; rows
// beyond nrows are clamped (their products are never stored)
constexpr int ROW_LOADS = 256 / (8 * G_WAVES);      // 8 rows per wavefront-wide load
struct RowTileLoader {
    const uint8_t* base;                            // first row of the tile (wave-uniform, lives in SGPRs)
    uint32_t off[ROW_LOADS];                        // this lane's byte offset from it, per load
    __device__ void init(const uint8_t* mat, int64_t ld, int64_t row0, int64_t nrows, int wave)
    {
        const int lane = fresh_lane();
        base = mat + row0 * ld;
        const int64_t left = nrows - row0;             // rows of the matrix from row0 on (>= 1)
        const int last = left > 255 ? 255 : (int)left - 1;
        const uint32_t ld32 = (uint32_t)ld;             // 256 rows x ld fits 32 bits (row bytes <= 2^23)
#pragma unroll
        for (int i = 0; i < ROW_LOADS; ++i) {
            const int row = (i * G_WAVES + wave) * 8 + (lane >> 3);
            const int lc = (lane & 7) ^ swz(row);
            off[i] = (uint32_t)(row < last ? row : last) * ld32 + lc * 16;
        }
    }
    __device__ void issue_one(int i, int64_t k0, uint8_t* lds_tile, int wave) const
    {
        lds_dma16(base + k0, off[i], lds_tile + (i * G_WAVES + wave) * 8 * ROWB);
    }
    __device__ void issue(int64_t k0, uint8_t* lds_tile, int wave) const
    {
#pragma unroll
        for (int i = 0; i < ROW_LOADS; ++i) issue_one(i, k0, lds_tile, wave);
    }
};

// operand reads [first, last) that go behind matrix instruction i of 8 when `parts` reads are spread evenly
__device__ constexpr int part_begin(int i, int parts) { return (i * parts + 7) / 8; }

constexpr std::integral_constant<int, 0> no_loads{};
constexpr std::integral_constant<int, 1> first_half{};
constexpr std::integral_constant<int, 2> second_half{};
constexpr std::integral_constant<int, 0> even{};
constexpr std::integral_constant<int, 1> odd{};

// ---- dense: Y = Xq . Wq^T ----------------------------------------------------------------------------
// Units of 128 k-bytes (128 / DENSE_SUB sub-steps); rings of two units per operand.  Kb = bytes per row.
constexpr int D_UNIT = BO * ROWB;                   // 32 KB, same for A and B
constexpr int SW_BYTES = BO * 4;                     // the tile's 256 channel scales; two copies (this tile, next tile)
constexpr int D_SW_OFF = 4 * D_UNIT;
constexpr int D_LDS = D_SW_OFF + 2 * SW_BYTES;      // 130 KB

template <int DT>
__global__ __launch_bounds__(G_THREADS) void k_dense(const uint8_t* __restrict__ Xq, const float* __restrict__ s_x, const uint8_t* __restrict__ Wq,
                                                     const float* __restrict__ s_w, int64_t M, int64_t O, int64_t Kb, uint16_t* __restrict__ Y,
                                                     int64_t ldy, int tiles_o, int tiles_t)
{
    typedef Mma<DT> MM;
    typedef typename MM::dfrag_t frag_t;
    constexpr int SUB = MM::DENSE_SUB, NSUB = ROWB / SUB, RPF = SUB / 32;    // k-bytes, sub-steps per unit, 16-byte reads per fragment
    constexpr int NPARTS = (4 + NBF) * RPF;
    struct Frags { frag_t a[4]; frag_t b[2][NBF]; };   // weights single-buffered, tokens double-buffered by sub-step parity
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave id in an SGPR
    const int wo = wave & 1, wt = wave >> 1;
    const int row = lane & 31, q = lane >> 5;
    const int nunits = (int)(Kb / ROWB);
    int arow[4], brow[NBF];
#pragma unroll
    for (int f = 0; f < 4; ++f) arow[f] = wo * 128 + panel_row(f, row);
#pragma unroll
    for (int bb = 0; bb < NBF; ++bb) brow[bb] = wt * (32 * NBF) + bb * 32 + row;

    // Per-tile state of the loaders.  It is set up for the next tile before the current tile's epilogue, so that
    // the first unit of the next tile is already in flight while the results are written out.
    RowTileLoader la, lb;
    int64_t o_blk = 0, t_blk = 0;
    auto setup_tile = [&](int to, int tt) {
        o_blk = (int64_t)to * BO;
        t_blk = (int64_t)tt * BT;
        la.init(Wq, Kb, o_blk, O, wave);
        lb.init(Xq, Kb, t_blk, M, wave);
    };
    // direct load number j (0..7) of this wavefront for a unit: weight and token rows alternate
    auto issue_part = [&](int unit, int j) {
        if (j & 1) lb.issue_one(j >> 1, (int64_t)unit * ROWB, smem + 2 * D_UNIT + (unit & 1) * D_UNIT, wave);
        else la.issue_one(j >> 1, (int64_t)unit * ROWB, smem + (unit & 1) * D_UNIT, wave);
    };
    auto issue = [&](int unit) {
#pragma unroll
        for (int j = 0; j < 2 * ROW_LOADS; ++j) issue_part(unit, j);
    };
    // one more direct load per wavefront with unit 0 of a tile: its channel scales (4 bytes a lane; waves 4..7
    // repeat what waves 0..3 fetch, so that every wavefront has the same number of loads in flight)
    auto issue_scales = [&](int parity) {
        if constexpr (MM::SCALED) {
            const int64_t o_first = o_blk + (wave & 3) * 64, left = O - 1 - o_first;     // clamp to the last channel
            const int left32 = left > 63 ? 63 : (int)left, ln = fresh_lane();
            const uint32_t oc = left32 < 0 ? 0u : (uint32_t)(ln < left32 ? ln : left32);
            lds_dma4(reinterpret_cast<const uint8_t*>(s_w + (left < 0 ? O - 1 : o_first)), oc * 4, smem + D_SW_OFF + parity * SW_BYTES + (wave & 3) * 256);
        }
    };
        // The epilogue stages in the second ring slot of either operand (waves 0..3 in A's, 4..7 in B's), so the first
    // slots can take unit 0 of the next tile while the epilogue runs.
    uint8_t* const stage = smem + (wave < 4 ? D_UNIT : 3 * D_UNIT) + (wave & 3) * EP_WAVE_BYTES;

    int to, tt;
    bool have = tile_of_round(0, tiles_o, tiles_t, to, tt);
    if (have) { setup_tile(to, tt); issue(0); issue_scales(0); }
    for (int round = 0; have; ++round) {
        typename MM::acc_t acc[4][NBF];
        zero_acc(acc);
        Frags R;
        // one 16-byte operand read of sub-step t (t counts sub-steps of the whole k range): fragment
        // part / RPF (0..3 weights, then tokens), piece part % RPF
        auto read_part = [&](int t, int part, int buf) {
            const uint8_t* sa = smem + ((t / NSUB) & 1) * D_UNIT;
            const int frag = part / RPF, piece = part % RPF;
            const int lc = (t % NSUB) * (SUB / 16) + q * RPF + piece;
            const v4i v = frag < 4 ? *tile_chunk(sa, arow[frag], lc) : *tile_chunk(sa + 2 * D_UNIT, brow[frag - 4], lc);
            frag_t& dst = frag < 4 ? R.a[frag] : R.b[buf][frag - 4];
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[4 * piece + e] = v[e];
        };
        // Sub-step t: its eight matrix instructions, with the operand reads of sub-step t+1 (if prefetch)
        // and, for loads = 1 / 2, the first / second four direct loads of unit `lunit` placed one by one
        // behind them.  A weight fragment is used by two consecutive instructions and refilled for the next
        // sub-step right behind the second; the token fragments of the next sub-step go to the other buffer.
        auto sub_step = [&](int t, auto parity, auto prefetch, auto loads, int lunit) {
            constexpr int cb = decltype(parity)::value;     // t & 1, known at every call site
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 4 * NBF; ++i) {
                acc[i / NBF][i % NBF] = MM::dense(R.a[i / NBF], R.b[cb][i % NBF], acc[i / NBF][i % NBF]);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (decltype(loads)::value > 0) {
                    if (i & 1) { issue_part(lunit, 4 * (decltype(loads)::value - 1) + (i >> 1)); __builtin_amdgcn_sched_barrier(0); }
                }
                if constexpr (decltype(prefetch)::value) {
                    if (i & 1) {
#pragma unroll
                        for (int piece = 0; piece < RPF; ++piece) read_part(t + 1, (i >> 1) * RPF + piece, cb ^ 1);
                    } else {
#pragma unroll
                        for (int part = part_begin(i, NBF * RPF); part < part_begin(i + 2, NBF * RPF); ++part) read_part(t + 1, 4 * RPF + part, cb ^ 1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        // the sub-steps of a unit except its last one; the first carries the second half of the loads of `lunit`
        auto unit_head = [&](int t, auto loads, int lunit) {
            static_assert(NSUB == 2 || NSUB == 4, "sub-steps per unit");
            sub_step(t, even, std::true_type{}, loads, lunit);
            if constexpr (NSUB == 4) {
                sub_step(t + 1, odd, std::true_type{}, no_loads, 0);
                sub_step(t + 2, even, std::true_type{}, no_loads, 0);
            }
        };

        // Unit u+2 is requested into the ring slot of unit u once every wavefront holds the operands of
        // the last sub-step of unit u (half of the loads ride on that sub-step, half on the next one), and
        // is awaited before the last sub-step of unit u+1.
        if (round > 0) wg_barrier();                  // epilogue staging of the previous tile has been read out
        if (nunits > 1) issue(1);
        // unit 0 was requested before the previous epilogue, whose stores sit between it and unit 1
        if (nunits > 1) wait_vmcnt<2 * ROW_LOADS>(); else wait_vmcnt<0>();
        wg_barrier();                                 // unit 0 (and the channel scales) are published
#pragma unroll
        for (int part = 0; part < NPARTS; ++part) read_part(0, part, 0);
        int t = 0, u = 0;
        unit_head(t, no_loads, 0);
        for (; u + 2 < nunits; ++u, t += NSUB) {      // unit u+1 is in flight, unit u+2 gets requested
            wait_vmcnt<0>();                          // unit u+1 has landed (and the reads of the last sub-step have returned)
            wg_barrier();                             // ... for every wavefront; nobody reads unit u's slot any more
            sub_step(t + NSUB - 1, odd, std::true_type{}, first_half, u + 2);
            unit_head(t + NSUB, second_half, u + 2);
        }
        if (u + 1 < nunits) {                         // the last unit follows without further requests
            wait_vmcnt<0>();
            wg_barrier();
            sub_step(t + NSUB - 1, odd, std::true_type{}, no_loads, 0);
            unit_head(t + NSUB, no_loads, 0);
            t += NSUB;
        }
        // this sub-tile of Y and its token scales (requested here: they arrive behind the last matrix instructions)
        const int64_t o_sub = o_blk + wo * 128, t_sub = t_blk + wt * (32 * NBF);
        const int64_t rows = M - t_sub, cols = O - o_sub;          // <= 0: nothing of this sub-tile exists
        const bool any = rows > 0 && cols > 0;
        const int rows_left = any ? (int)(rows > 64 ? 64 : rows) : 0, cols_left = any ? (int)(cols > 128 ? 128 : cols) : 0;
        float sx[NBF];
        load_token_scales<MM::SCALED>(sx, MM::SCALED && any ? s_x + t_sub : s_x, rows_left);
        sub_step(t + NSUB - 1, odd, std::false_type{}, no_loads, 0);
        wg_barrier();                                 // every wave is done with the operand tiles: LDS becomes staging
        uint16_t* const Y_sub = any ? Y + t_sub * ldy + o_sub : Y;
        settle(sx);                                   // the token scales have arrived: no wait for them behind the loads requested next
        have = tile_of_round(round + 1, tiles_o, tiles_t, to, tt);
        if (have) { setup_tile(to, tt); issue(0); issue_scales((round + 1) & 1); }
        store_tile<MM::SCALED, 32, false>(acc, sx, reinterpret_cast<const float*>(smem + D_SW_OFF + (round & 1) * SW_BYTES) + wo * 128, Y_sub,
                                   (uint32_t)ldy, rows_left, cols_left, stage);
    }
}

// ---- sparse over the lifted width: Y = X' . W'^T, W' packed 2:4 -------------------------------------
// Sub-step = 64 lifted bytes (one sparse matrix instruction deep); unit = two sub-steps = 128 lifted
// bytes.  Ring of three units; a unit is a 32 KB token tile (128-byte rows), 16 KB of weight values
// [panel 2][sub-step 2][fragment 4][lane 64][16 B] and 4 KB of index words
// [panel 2][sub-step 2][lane 64][fragment 4][4 B], both in the order slide_decompose stores them.
// Kpb = bytes per lifted row.
constexpr int S_RING = 3;
constexpr int S_B_UNIT = BT * ROWB;                 // 32 KB
constexpr int S_AV_UNIT = BO * 64;                  // 16 KB
constexpr int S_AM_UNIT = BO * 16;                  // 4 KB
constexpr int S_AV_OFF = S_RING * S_B_UNIT;
constexpr int S_AM_OFF = S_AV_OFF + S_RING * S_AV_UNIT;
constexpr int S_SW_OFF = S_AM_OFF + S_RING * S_AM_UNIT;
constexpr int S_LDS = S_SW_OFF + 2 * SW_BYTES;      // 158 KB
constexpr int EP_BYTES = G_WAVES * EP_WAVE_BYTES;   // 64 KB of staging
static_assert(S_LDS <= 160 * 1024 && EP_BYTES <= 2 * S_B_UNIT && EP_WAVE_BYTES * 4 <= D_UNIT, "LDS budget");
constexpr int S_LPU = ROW_LOADS + 2 + 2;            // direct loads per wavefront and unit: token rows, values, index words

// weight values single-buffered; index words and token fragments double-buffered by sub-step parity
struct SparseFrags { v4i a[4]; v4i idx[2]; v8i b[2][NBF]; };

template <int DT>
__global__ __launch_bounds__(G_THREADS) void k_sparse(const uint8_t* __restrict__ XL, const float* __restrict__ s_x, const uint8_t* __restrict__ w_vals,
                                                      const uint8_t* __restrict__ w_meta, const float* __restrict__ s_w, int64_t M, int64_t O,
                                                      int64_t Kpb, uint16_t* __restrict__ Y, int64_t ldy, int tiles_o, int tiles_t)
{
    typedef Mma<DT> MM;
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave id in an SGPR
    const int wo = wave & 1, wt = wave >> 1;
    const int n = lane & 31, qb = lane >> 5;
    const int U = (int)(Kpb / (2 * FRAG_KB));         // units
    const int64_t npanels = (O + PANEL - 1) / PANEL;
    int brow[NBF];
#pragma unroll
    for (int bb = 0; bb < NBF; ++bb) brow[bb] = wt * (32 * NBF) + bb * 32 + n;

    // Per-tile state of the loaders.  It is set up for the next tile before the current tile's epilogue, so that
    // the first unit of the next tile is already in flight while the results are written out.
    RowTileLoader lb;
    const uint8_t *av_src = nullptr, *am_src = nullptr;
    int64_t o_blk = 0, t_blk = 0;
    const int piece = (wave & 3) * 2;
    uint8_t* const av_dst = smem + S_AV_OFF + (wave >> 2) * 8192 + piece * 1024;
    uint8_t* const am_dst = smem + S_AM_OFF + (wave >> 2) * 2048 + piece * 256;
    const uint32_t lane16 = lane * 16, lane4 = lane * 4;
    // Packed weights: per 128-channel panel the two sub-steps of a unit are contiguous, 8 KB of values
    // and 2 KB of index words.  Waves 0..3 fetch panel 2*to, waves 4..7 panel 2*to+1 (clamped to the last
    // panel; a clamped panel only feeds rows that are never stored): two 1 KB pieces of values (16 bytes
    // a lane) and two 256-byte pieces of index words (4 bytes a lane) each.
    auto setup_tile = [&](int to, int tt) {
        o_blk = (int64_t)to * BO;
        t_blk = (int64_t)tt * BT;
        lb.init(XL, Kpb, t_blk, M, wave);
        int64_t panel = (int64_t)to * 2 + (wave >> 2);
        panel = panel < npanels ? panel : npanels - 1;
        av_src = w_vals + panel * U * 8192 + piece * 1024;     // wave-uniform
        am_src = w_meta + panel * U * 2048 + piece * 256;
    };
    // direct load number j (0..7) of this wavefront for unit u: token rows, values, token rows, index words, twice
    auto issue_part = [&](int u, int slot, int j) {
        const int half = j >> 2;
        if (!(j & 1)) lb.issue_one(j >> 1, (int64_t)u * ROWB, smem + slot * S_B_UNIT, wave);
        else if ((j & 3) == 1) lds_dma16(av_src + (int64_t)u * 8192 + half * 1024, lane16, av_dst + slot * S_AV_UNIT + half * 1024);
        else lds_dma4(am_src + (int64_t)u * 2048 + half * 256, lane4, am_dst + slot * S_AM_UNIT + half * 256);
    };
    auto issue = [&](int u, int slot) {
#pragma unroll
        for (int j = 0; j < S_LPU; ++j) issue_part(u, slot, j);
    };
    // one more direct load per wavefront with unit 0 of a tile: its channel scales (4 bytes a lane; waves 4..7
    // repeat what waves 0..3 fetch, so that every wavefront has the same number of loads in flight)
    auto issue_scales = [&](int parity) {
        if constexpr (MM::SCALED) {
            const int64_t o_first = o_blk + (wave & 3) * 64, left = O - 1 - o_first;     // clamp to the last channel
            const int left32 = left > 63 ? 63 : (int)left, ln = fresh_lane();
            const uint32_t oc = left32 < 0 ? 0u : (uint32_t)(ln < left32 ? ln : left32);
            lds_dma4(reinterpret_cast<const uint8_t*>(s_w + (left < 0 ? O - 1 : o_first)), oc * 4, smem + S_SW_OFF + parity * SW_BYTES + (wave & 3) * 256);
        }
    };

    // Unit u of a tile lives in ring slot (u + 2) % 3: the epilogue's staging area is the token part of
    // slots 0 and 1, so slot 2 (and the weight parts of all slots) can take the next tile's first unit
    // while the epilogue runs.
    int to, tt;
    bool have = tile_of_round(0, tiles_o, tiles_t, to, tt);
    if (have) { setup_tile(to, tt); issue(0, 2); issue_scales(0); }
    for (int round = 0; have; ++round) {
        typename MM::acc_t acc[4][NBF];
        zero_acc(acc);
        SparseFrags R;
        // one operand read of half h of the unit in ring slot `slot`: parts 0..3 weight values, 4 their
        // index words, 5..8 the two halves of the two token fragments
        auto read_part = [&](int slot, int h, int part) {
            if (part < 4) R.a[part] = *reinterpret_cast<const v4i*>(smem + S_AV_OFF + slot * S_AV_UNIT + ((wo * 2 + h) * 4 + part) * 1024 + lane16);
            else if (part == 4) R.idx[h] = *reinterpret_cast<const v4i*>(smem + S_AM_OFF + slot * S_AM_UNIT + (wo * 2 + h) * 1024 + lane16);
            else {
                const int bb = (part - 5) >> 1, hh = (part - 5) & 1;
                const v4i v = *tile_chunk(smem + slot * S_B_UNIT, brow[bb], 4 * h + 2 * qb + hh);
#pragma unroll
                for (int e = 0; e < 4; ++e) R.b[h][bb][4 * hh + e] = v[e];
            }
        };
        // Sub-step h^1 of a unit: eight matrix instructions, with the nine operand reads of the following
        // sub-step (half h of the unit in `slot`) and, for loads = 1 / 2, the first / second four direct
        // loads of unit `lunit` (into ring slot lslot) placed one by one behind them.  A weight fragment is
        // used by two consecutive instructions and refilled right behind the second; index words and token
        // fragments of the following sub-step go to the other buffer.
        auto sub_step = [&](int slot, int h, auto prefetch, auto loads, int lunit, int lslot) {
            const int c = h ^ 1;                      // buffers of the sub-step being computed
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 4 * NBF; ++i) {
                acc[i / NBF][i % NBF] = MM::sparse(R.a[i / NBF], R.b[c][i % NBF], acc[i / NBF][i % NBF], R.idx[c][i / NBF]);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (decltype(loads)::value > 0) {
                    if (i & 1) { issue_part(lunit, lslot, 4 * (decltype(loads)::value - 1) + (i >> 1)); __builtin_amdgcn_sched_barrier(0); }
                }
                if constexpr (decltype(prefetch)::value) {
                    if (i & 1) read_part(slot, h, i >> 1); else read_part(slot, h, 5 + (i >> 1));
                    if (i == 1) read_part(slot, h, 4);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };

        // The two wavefronts of a SIMD run freely against each other; the workgroup meets once per unit.
        // Before that barrier a wavefront holds the operands of the unit's second sub-step in registers and
        // has seen its own loads of the next unit land; after it nobody reads the unit's ring slot any more,
        // so the unit three ahead is requested into it, and the next unit is visible to everybody.
        if (round > 0) wg_barrier();                  // epilogue staging of the previous tile has been read out
        if (U > 1) issue(1, 0);
        if (U > 2) issue(2, 1);
        // unit 0 was requested before the previous epilogue, whose stores sit between it and units 1 and 2
        if (U > 2) wait_vmcnt<2 * S_LPU>(); else if (U > 1) wait_vmcnt<S_LPU>(); else wait_vmcnt<0>();
        wg_barrier();                                 // unit 0 (and the channel scales) are published
#pragma unroll
        for (int part = 0; part < 9; ++part) read_part(2, 0, part);
        constexpr std::true_type prefetch{};
        int u = 0, slot = 2;
        sub_step(slot, 1, prefetch, no_loads, 0, 0);
        for (; u + 3 < U; ++u) {                      // units u+1 and u+2 are in flight, unit u+3 gets requested
            const int nslot = slot == S_RING - 1 ? 0 : slot + 1;
            wait_vmcnt<S_LPU>();                      // own loads of unit u+1 have landed, own reads of unit u have returned
            wg_barrier();
            sub_step(nslot, 0, prefetch, first_half, u + 3, slot);
            sub_step(nslot, 1, prefetch, second_half, u + 3, slot);
            slot = nslot;
        }
        for (; u + 1 < U; ++u) {                      // nothing left to request
            const int nslot = slot == S_RING - 1 ? 0 : slot + 1;
            wait_vmcnt<0>();
            wg_barrier();
            sub_step(nslot, 0, prefetch, no_loads, 0, 0);
            sub_step(nslot, 1, prefetch, no_loads, 0, 0);
            slot = nslot;
        }
        // this sub-tile of Y and its token scales (requested here: they arrive behind the last matrix instructions)
        const int64_t o_sub = o_blk + wo * 128, t_sub = t_blk + wt * (32 * NBF);
        const int64_t rows = M - t_sub, cols = O - o_sub;          // <= 0: nothing of this sub-tile exists
        const bool any = rows > 0 && cols > 0;
        const int rows_left = any ? (int)(rows > 64 ? 64 : rows) : 0, cols_left = any ? (int)(cols > 128 ? 128 : cols) : 0;
        float sx[NBF];
        load_token_scales<MM::SCALED>(sx, MM::SCALED && any ? s_x + t_sub : s_x, rows_left);
        sub_step(slot, 0, std::false_type{}, no_loads, 0, 0);
        wg_barrier();                                 // every wave is done with the operand tiles: LDS becomes staging
        uint16_t* const Y_sub = any ? Y + t_sub * ldy + o_sub : Y;
        settle(sx);                                   // the token scales have arrived: no wait for them behind the loads requested next
        have = tile_of_round(round + 1, tiles_o, tiles_t, to, tt);
        if (have) { setup_tile(to, tt); issue(0, 2); issue_scales((round + 1) & 1); }
        store_tile<MM::SCALED, 32, false>(acc, sx, reinterpret_cast<const float*>(smem + S_SW_OFF + (round & 1) * SW_BYTES) + wo * 128, Y_sub,
                                   (uint32_t)ldy, rows_left, cols_left, smem + wave * EP_WAVE_BYTES);
    }
}

}  // namespace ss

using namespace ss;

// one persistent workgroup per compute unit of the current device (fewer if there are fewer tiles)
static int persistent_grid(int ntiles)
{
    const int cus = cu_count();
    return ntiles < cus ? ntiles : cus;
}

static ss_status check_gemm(const void* X, const float* s_x, const void* W, const float* s_w, int64_t M, int64_t O, int64_t K,
                            ss_dtype dtype, const void* Y, int64_t ldy)
{
    if (!valid_dtype(dtype)) return SS_ERR_DTYPE;
    if (M < 0 || O < 0 || K <= 0 || (K * elem_size(dtype)) % KSTEP != 0 || ldy < O || M > (1 << 24) || ldy >= (1 << 22) || K * elem_size(dtype) > (1 << 23))
        return SS_ERR_SHAPE;
    if (M == 0 || O == 0) return SS_OK;
    if (!X || !W || !Y) return SS_ERR_NULL;
    if (!unscaled(dtype) && (!s_x || !s_w)) return SS_ERR_NULL;
    if (((uintptr_t)X & 15) || ((uintptr_t)W & 15)) return SS_ERR_SHAPE;
    return SS_OK;
}

template <int DT>
static ss_status launch_dense(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, void* Y,
                              int64_t ldy, int tiles_o, int tiles_t, int grid, hipStream_t stream)
{
    if (allow_dynamic_lds<k_dense<DT>>(D_LDS) != SS_OK) return SS_ERR_HIP;
    hipLaunchKernelGGL((k_dense<DT>), dim3(grid), dim3(G_THREADS), D_LDS, stream, static_cast<const uint8_t*>(Xq), s_x,
                       static_cast<const uint8_t*>(Wq), s_w, M, O, Kb, static_cast<uint16_t*>(Y), ldy, tiles_o, tiles_t);
    return launch_status();
}

template <int DT>
static ss_status launch_sparse(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                               int64_t Kpb, void* Y, int64_t ldy, int tiles_o, int tiles_t, int grid, hipStream_t stream)
{
    if (allow_dynamic_lds<k_sparse<DT>>(S_LDS) != SS_OK) return SS_ERR_HIP;
    hipLaunchKernelGGL((k_sparse<DT>), dim3(grid), dim3(G_THREADS), S_LDS, stream, static_cast<const uint8_t*>(XL), s_x,
                       static_cast<const uint8_t*>(w_vals), static_cast<const uint8_t*>(w_meta), s_w, M, O, Kpb, static_cast<uint16_t*>(Y), ldy,
                       tiles_o, tiles_t);
    return launch_status();
}

// 256 x 256 tile kernels (arguments already validated)
namespace ss {

ss_status launch_dense_tile(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t Kb, ss_dtype dtype,
                            void* Y, int64_t ldy, hipStream_t hs)
{
    const int tiles_o = (int)((O + BO - 1) / BO), tiles_t = (int)((M + BT - 1) / BT);
    const int grid = persistent_grid(tiles_o * tiles_t);
    if (grid <= 0) return SS_ERR_HIP;
    switch (dtype) {
    case SS_I8: return launch_dense<SS_I8>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, tiles_o, tiles_t, grid, hs);
    case SS_FP8_E4M3: return launch_dense<SS_FP8_E4M3>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, tiles_o, tiles_t, grid, hs);
    case SS_BF16: return launch_dense<SS_BF16>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, tiles_o, tiles_t, grid, hs);
    case SS_FP16: return launch_dense<SS_FP16>(Xq, s_x, Wq, s_w, M, O, Kb, Y, ldy, tiles_o, tiles_t, grid, hs);
    }
    return SS_ERR_DTYPE;
}

ss_status launch_sparse_tile(const void* XL, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w, int64_t M, int64_t O,
                             int64_t Kpb, ss_dtype dtype, void* Y, int64_t ldy, hipStream_t hs)
{
    const int tiles_o = (int)((O + BO - 1) / BO), tiles_t = (int)((M + BT - 1) / BT);
    const int grid = persistent_grid(tiles_o * tiles_t);
    if (grid <= 0) return SS_ERR_HIP;
    switch (dtype) {
    case SS_I8: return launch_sparse<SS_I8>(XL, s_x, w_vals, w_meta, s_w, M, O, Kpb, Y, ldy, tiles_o, tiles_t, grid, hs);
    case SS_FP8_E4M3: return launch_sparse<SS_FP8_E4M3>(XL, s_x, w_vals, w_meta, s_w, M, O, Kpb, Y, ldy, tiles_o, tiles_t, grid, hs);
    case SS_BF16: return launch_sparse<SS_BF16>(XL, s_x, w_vals, w_meta, s_w, M, O, Kpb, Y, ldy, tiles_o, tiles_t, grid, hs);
    case SS_FP16: return launch_sparse<SS_FP16>(XL, s_x, w_vals, w_meta, s_w, M, O, Kpb, Y, ldy, tiles_o, tiles_t, grid, hs);
    }
    return SS_ERR_DTYPE;
}

}  // namespace ss

static ss_status check_workspace(const void* workspace, size_t workspace_bytes)
{
    if (workspace_bytes > 0 && !workspace) return SS_ERR_NULL;
    if ((uintptr_t)workspace & 15) return SS_ERR_WORKSPACE;
    return SS_OK;
}

extern "C" size_t slide_gemm_workspace_bytes(int64_t M, int64_t O, int64_t K, ss_dtype dtype)
{
    if (!valid_dtype(dtype) || M <= 0 || O <= 0 || K <= 0 || (K * elem_size(dtype)) % KSTEP != 0) return 0;
    const int64_t units = K * elem_size(dtype) / KSTEP;
    const ss_plan p = plan_gemm(M, O, units, (size_t)-1);
    if (p.path == SS_PATH_MID) return mid_workspace_bytes(M, O, p.S);
    return p.path == SS_PATH_SKINNY ? skinny_workspace_bytes(M, O, p.S) : 0;
}

extern "C" ss_status dense_gemm_ws(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t K,
                                   ss_dtype dtype, void* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream)
{
    ss_status st = check_gemm(Xq, s_x, Wq, s_w, M, O, K, dtype, Y, ldy);
    if (st == SS_OK) st = check_workspace(workspace, workspace_bytes);
    if (st != SS_OK || M == 0 || O == 0) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int64_t Kb = K * elem_size(dtype);
    const ss_plan p = plan_gemm(M, O, Kb / KSTEP, workspace_bytes);
    if (p.path == SS_PATH_SKINNY) return launch_dense_skinny(Xq, s_x, Wq, s_w, M, O, Kb, dtype, Y, ldy, workspace, p.S, hs);
    if (p.path == SS_PATH_MID) return launch_dense_mid(Xq, s_x, Wq, s_w, M, O, Kb, dtype, Y, ldy, workspace, p.S, hs);
    return launch_dense_tile(Xq, s_x, Wq, s_w, M, O, Kb, dtype, Y, ldy, hs);
}

extern "C" ss_status dense_gemm(const void* Xq, const float* s_x, const void* Wq, const float* s_w, int64_t M, int64_t O, int64_t K,
                                ss_dtype dtype, void* Y, int64_t ldy, void* stream)
{
    return dense_gemm_ws(Xq, s_x, Wq, s_w, M, O, K, dtype, Y, ldy, nullptr, 0, stream);
}

extern "C" ss_status slide_sparse_gemm_ws(const void* X_lifted, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w,
                                          int64_t M, int64_t O, int64_t K_lifted, ss_dtype dtype, void* Y, int64_t ldy, void* workspace,
                                          size_t workspace_bytes, void* stream)
{
    ss_status st = check_gemm(X_lifted, s_x, w_vals, s_w, M, O, K_lifted, dtype, Y, ldy);
    if (st == SS_OK) st = check_workspace(workspace, workspace_bytes);
    if (st != SS_OK || M == 0 || O == 0) return st;
    if (!w_meta) return SS_ERR_NULL;
    if ((uintptr_t)w_meta & 15) return SS_ERR_SHAPE;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int64_t Kpb = K_lifted * elem_size(dtype);
    const ss_plan p = plan_gemm(M, O, Kpb / KSTEP, workspace_bytes);
    if (p.path == SS_PATH_SKINNY) return launch_sparse_skinny(X_lifted, s_x, w_vals, w_meta, s_w, M, O, Kpb, dtype, Y, ldy, workspace, p.S, hs);
    if (p.path == SS_PATH_MID) return launch_sparse_mid(X_lifted, s_x, w_vals, w_meta, s_w, M, O, Kpb, dtype, Y, ldy, workspace, p.S, hs);
    return launch_sparse_tile(X_lifted, s_x, w_vals, w_meta, s_w, M, O, Kpb, dtype, Y, ldy, hs);
}

extern "C" ss_status slide_sparse_gemm(const void* X_lifted, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w,
                                       int64_t M, int64_t O, int64_t K_lifted, ss_dtype dtype, void* Y, int64_t ldy, void* stream)
{
    return slide_sparse_gemm_ws(X_lifted, s_x, w_vals, w_meta, s_w, M, O, K_lifted, dtype, Y, ldy, nullptr, 0, stream);
}

// ---- entry point for callers that cannot allocate: the split-k scratch is a static device array ----------------
// 16 MiB: S k ranges x tiles of 128 x 128 x 4 bytes with S x tiles <= one workgroup per compute unit (256 x 64 KiB).
constexpr size_t SS_STATIC_SCRATCH_BYTES = 16u << 20;
static __device__ __align__(256) unsigned char scratch[SS_STATIC_SCRATCH_BYTES];

// Device address of this device's copy of `scratch`, looked up once per device with that device current (in host code
// the array's name is only a handle for the lookup, never a device address).
static ss_status static_scratch(void** ptr)
{
    static std::atomic<void*> known[MAX_TRACKED_DEVICES];
    const int d = current_device();
    if (d < 0 || d >= MAX_TRACKED_DEVICES) return SS_ERR_HIP;
    void* p = known[d].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SS_ERR_HIP;
        known[d].store(p, std::memory_order_release);
    }
    *ptr = p;
    return SS_OK;
}

extern "C" size_t slide_static_scratch_bytes(void) { return SS_STATIC_SCRATCH_BYTES; }

extern "C" ss_status slide_sparse_gemm_static(const void* X_lifted, const float* s_x, const void* w_vals, const void* w_meta, const float* s_w,
                                              int64_t M, int64_t O, int64_t K_lifted, ss_dtype dtype, void* Y, int64_t ldy, void* stream)
{
    ss_status st = check_gemm(X_lifted, s_x, w_vals, s_w, M, O, K_lifted, dtype, Y, ldy);
    if (st != SS_OK || M == 0 || O == 0) return st;
    if (!w_meta) return SS_ERR_NULL;
    if ((uintptr_t)w_meta & 15) return SS_ERR_SHAPE;
    // what the shape would use with an unlimited workspace must fit the static array
    if (slide_gemm_workspace_bytes(M, O, K_lifted, dtype) > SS_STATIC_SCRATCH_BYTES) return SS_ERR_SCRATCH;
    void* ws = nullptr;
    st = static_scratch(&ws);
    if (st != SS_OK) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int64_t Kpb = K_lifted * elem_size(dtype);
    const ss_plan p = plan_gemm(M, O, Kpb / KSTEP, SS_STATIC_SCRATCH_BYTES);
    if (p.path == SS_PATH_SKINNY) return launch_sparse_skinny(X_lifted, s_x, w_vals, w_meta, s_w, M, O, Kpb, dtype, Y, ldy, ws, p.S, hs);
    if (p.path == SS_PATH_MID) return launch_sparse_mid(X_lifted, s_x, w_vals, w_meta, s_w, M, O, Kpb, dtype, Y, ldy, ws, p.S, hs);
    return launch_sparse_tile(X_lifted, s_x, w_vals, w_meta, s_w, M, O, Kpb, dtype, Y, ldy, hs);
}

extern "C" const char* ss_status_string(ss_status s)
{
    switch (s) {
    case SS_OK: return "ok";
    case SS_ERR_NULL: return "null pointer";
    case SS_ERR_BAD_PATTERN_N: return "pattern parameter N outside 2..8";
    case SS_ERR_SHAPE: return "bad shape, stride or alignment";
    case SS_ERR_DTYPE: return "unsupported dtype";
    case SS_ERR_WORKSPACE: return "workspace not 16-byte aligned";
    case SS_ERR_HIP: return "HIP runtime error";
    case SS_ERR_SCRATCH: return "shape needs more scratch memory than the static buffer holds (slide_static_scratch_bytes)";
    }
    return "unknown status";
}

extern "C" int slide_format_version(void) { return SS_FORMAT_VERSION; }
