// slide_decompose: Sliding Window Decomposition (Alg. 2, greedy residual allocation) fused
// with 2:4 compression, written output-oriented: one thread produces one lane's worth of
// sparse-operand registers (16 bytes of stored values + one index word), so every store is coalesced.
// A thread re-runs the greedy over the few earlier windows of the same 2N block to recover
// the carry; the block is at most 16 elements, so this costs a handful of integer ops.
#include "ss_common.h"
#include "packed_layout.h"

namespace ss {

template <int ES> struct Elem;
template <> struct Elem<1> { typedef uint8_t T; __device__ static bool nz(T v, bool fp) { return fp ? (v & 0x7F) != 0 : v != 0; } };
template <> struct Elem<2> { typedef uint16_t T; __device__ static bool nz(T v, bool) { return (v & 0x7FFF) != 0; } };

// One window of the decomposition: values and positions (i0 < i1) of window l of block g of a
// row, plus the block's non-zero count.  `row` points at the row's first element, K is its
// length: elements at and beyond K read as zero (last block completed with zeros, Alg. 1's
// n_g = ceil(K / 2N)), and a block at or beyond n_g is all zero (padding of the stored width).
template <int ES>
__device__ inline void slide_window(const typename Elem<ES>::T* row, int K, int N, int g, int l, bool fp,
                                    typename Elem<ES>::T& v0, typename Elem<ES>::T& v1, uint32_t& i0, uint32_t& i1, int& nnz)
{
    typedef typename Elem<ES>::T T;
    const T* blk = row + (int64_t)g * 2 * N;
    const int left = K - g * 2 * N;                      // elements of this block inside the row (may be <= 0)
    uint32_t nzmask = 0;
    for (int p = 0; p < 2 * l + 4; ++p) nzmask |= (uint32_t)(p < left && Elem<ES>::nz(blk[p], fp)) << p;
    uint32_t used = 0, taken = 0;
    for (int w = 0; w <= l; ++w) {                       // greedy, windows in ascending order
        int cnt = 0;
        taken = 0;
        for (int d = 0; d < 4; ++d) {
            const int p = 2 * w + d;
            if (((nzmask >> p) & 1u) && !((used >> p) & 1u) && cnt < 2) { used |= 1u << p; taken |= 1u << d; ++cnt; }
        }
    }
    if (l == 0) {                                        // pattern check, once per block
        uint32_t all = nzmask;
        for (int p = 4; p < 2 * N; ++p) all |= (uint32_t)(p < left && Elem<ES>::nz(blk[p], fp)) << p;
        nnz = __popc(all);
    } else nnz = 0;
    // pad to two positions with the lowest offsets that hold no stored non-zero
    uint32_t chosen = taken;
    for (int d = 0; d < 4 && __popc(chosen) < 2; ++d) chosen |= 1u << d;
    i0 = __ffs(chosen) - 1;
    i1 = 31 - __clz(chosen);
    v0 = ((taken >> i0) & 1u) ? blk[2 * l + i0] : (T)0;
    v1 = ((taken >> i1) & 1u) ? blk[2 * l + i1] : (T)0;
}

// canonical form: one thread per (row, window)
template <int ES>
__global__ __launch_bounds__(256) void k_decompose_canonical(const typename Elem<ES>::T* __restrict__ Wq, int64_t O, int K, int N, bool fp,
                                                              typename Elem<ES>::T* __restrict__ vals, uint8_t* __restrict__ idx,
                                                              int32_t* __restrict__ violations)
{
    const int nwin = (int)n_groups(K, N) * (N - 1);
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= O * nwin) return;
    const int64_t o = id / nwin;
    const int j = (int)(id - o * nwin);
    const int g = j / (N - 1), l = j - g * (N - 1);
    typename Elem<ES>::T v0, v1; uint32_t i0, i1; int nnz;
    slide_window<ES>(Wq + o * (int64_t)K, K, N, g, l, fp, v0, v1, i0, i1, nnz);
    vals[o * (int64_t)nwin * 2 + 2 * j] = v0;
    vals[o * (int64_t)nwin * 2 + 2 * j + 1] = v1;
    idx[o * (int64_t)nwin + j] = (uint8_t)(i0 | (i1 << 2));
    if (violations && nnz > 2 * N - 2) atomicAdd(violations, 1);
}

// One 2N block of a row with its decomposition: the block's elements (zero beyond the row), the positions each of
// its N-1 windows takes (Alg. 2, greedy in window order) and its non-zero count.  Loading and decomposing a block once
// and reading several windows from it is what the packed kernel does: a lane's windows come in runs of consecutive
// windows, so it touches two to four blocks instead of re-reading one per window.
template <int ES> struct SlideBlock {
    typedef typename Elem<ES>::T T;
    T v[16];
    uint32_t taken[7];                                   // per window: 4-bit mask of the offsets it stores
    int nnz;

    __device__ void load(const T* row, int K, int N, int g, bool fp)
    {
        const T* blk = row + (int64_t)g * 2 * N;
        const int left = K - g * 2 * N;                  // elements of this block inside the row (<= 0: none)
        constexpr int PER = 4 / ES;                      // elements per 32-bit word
        if (left >= 2 * N && (((uintptr_t)blk) & 3) == 0 && ((2 * N) % PER) == 0) {
            const uint32_t* w = reinterpret_cast<const uint32_t*>(blk);
#pragma unroll
            for (int i = 0; i < 16 / PER; ++i) {
                const uint32_t x = i * PER < 2 * N ? w[i] : 0u;
#pragma unroll
                for (int e = 0; e < PER; ++e) v[i * PER + e] = (T)(x >> (8 * ES * e));
            }
        } else {
#pragma unroll
            for (int p = 0; p < 16; ++p) v[p] = (p < 2 * N && p < left) ? blk[p] : (T)0;
        }
        uint32_t nzmask = 0;
#pragma unroll
        for (int p = 0; p < 16; ++p) nzmask |= (uint32_t)(p < 2 * N && Elem<ES>::nz(v[p], fp)) << p;
        nnz = __popc(nzmask);
        uint32_t used = 0;
#pragma unroll
        for (int w = 0; w < 7; ++w) {                    // windows in ascending order; each takes its first <= 2 unused non-zeros
            uint32_t t = 0;
            int cnt = 0;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int p = 2 * w + d;
                if (w < N - 1 && ((nzmask >> p) & 1u) && !((used >> p) & 1u) && cnt < 2) { used |= 1u << p; t |= 1u << d; ++cnt; }
            }
            taken[w] = t;
        }
    }

    // window l: stored values and their positions i0 < i1 (padded with the lowest offsets that hold no stored non-zero)
    __device__ void window(int l, T& v0, T& v1, uint32_t& i0, uint32_t& i1) const
    {
        uint32_t t = 0;
#pragma unroll
        for (int w = 0; w < 7; ++w) t = w == l ? taken[w] : t;
        uint32_t chosen = t;
#pragma unroll
        for (int d = 0; d < 4; ++d) if (__popc(chosen) < 2) chosen |= 1u << d;
        i0 = __ffs(chosen) - 1;
        i1 = 31 - __clz(chosen);
        const int p0 = 2 * l + (int)i0, p1 = 2 * l + (int)i1;
        T e0 = 0, e1 = 0;
#pragma unroll
        for (int p = 0; p < 16; ++p) { e0 = p == p0 ? v[p] : e0; e1 = p == p1 ? v[p] : e1; }
        v0 = ((t >> i0) & 1u) ? e0 : (T)0;
        v1 = ((t >> i1) & 1u) ? e1 : (T)0;
    }
};

// packed form: one thread per (panel, 64-byte step, fragment, lane).  FUSED: the window order of the GEMM that lifts
// the activations itself (N = 4; fused_window in packed_layout.h) instead of the order of the lifted row.
template <int ES, bool FUSED>
__global__ __launch_bounds__(256) void k_decompose_packed(const typename Elem<ES>::T* __restrict__ Wq, int64_t O, int K, int N, bool fp,
                                                           uint4* __restrict__ vals, uint32_t* __restrict__ meta, int64_t nslots,
                                                           int nsteps, int32_t* __restrict__ violations)
{
    typedef typename Elem<ES>::T T;
    constexpr int NW = 8 / ES;                           // windows per lane
    const int64_t slot = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (slot >= nslots) return;
    const int lane = (int)(slot & 63);
    const int f = (int)((slot >> 6) & 3);
    const int64_t ps = slot >> 8;
    const int64_t panel = ps / nsteps;
    const int step = (int)(ps - panel * nsteps);
    const int64_t o = panel * PANEL + panel_row(f, lane & 31);
    const int qa = lane >> 5;
    uint32_t v[4] = {0, 0, 0, 0};
    uint32_t m = ES == 1 ? 0x44444444u : 0x4444u;        // positions (0, 1) everywhere: an all-zero fragment
    if (o < O) {
        m = 0;
        int bad = 0;
        SlideBlock<ES> B;
        int g_held = -1;
        const T* row = Wq + o * (int64_t)K;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            int g, l;
            if constexpr (FUSED) fused_window<ES>(step, qa, w, g, l);
            else {
                const int j = step * (2 * NW) + step_window<ES>(qa, w);
                g = j / (N - 1);
                l = j - g * (N - 1);
            }
            if (g != g_held) {                           // windows of one block are neighbours in a lane, so every block is loaded once
                B.load(row, K, N, g, fp);
                g_held = g;
            }
            T v0, v1; uint32_t i0, i1;
            B.window(l, v0, v1, i0, i1);
            if constexpr (ES == 1) v[w >> 1] |= ((uint32_t)v0 | ((uint32_t)v1 << 8)) << (16 * (w & 1));
            else v[w] = (uint32_t)v0 | ((uint32_t)v1 << 16);
            m |= (i0 | (i1 << 2)) << (4 * w);
            bad += (l == 0 && B.nnz > 2 * N - 2);       // pattern check, counted by the lane that holds the block's first window
        }
        if (violations && bad) atomicAdd(violations, bad);
    }
    vals[slot] = make_uint4(v[0], v[1], v[2], v[3]);
    meta[(ps * 64 + lane) * FRAGS_PER_PANEL + f] = m;   // index words lane-major: one 16-byte read gives a lane all four
}

}  // namespace ss

using namespace ss;

static ss_status check_decompose(int64_t O, int64_t K, int N, ss_dtype dtype)
{
    if (!valid_N(N)) return SS_ERR_BAD_PATTERN_N;
    if (!valid_dtype(dtype)) return SS_ERR_DTYPE;
    if (O < 0 || K <= 0 || K > (1 << 24) || O > (1 << 24)) return SS_ERR_SHAPE;
    return SS_OK;
}

extern "C" ss_status slide_packed_sizes(int64_t O, int64_t K, int N, ss_dtype dtype, size_t* vals_bytes, size_t* meta_bytes)
{
    ss_status st = check_decompose(O, K, N, dtype);
    if (st != SS_OK) return st;
    if (!vals_bytes || !meta_bytes) return SS_ERR_NULL;
    const int64_t Kpb = lifted_ld(K, N, elem_size(dtype)) * elem_size(dtype);    // stored bytes of a lifted row
    const int64_t Opad = (O + PANEL - 1) / PANEL * PANEL;
    *vals_bytes = (size_t)(Opad * (Kpb / 2));
    *meta_bytes = (size_t)(Opad * (Kpb / 8));            // one 4-byte index word per 16 bytes of values
    return SS_OK;
}

template <bool FUSED>
static ss_status launch_packed(const void* Wq, int64_t O, int64_t K, int N, ss_dtype dtype, int64_t Kpb, void* w_vals, void* w_meta,
                               int32_t* violations, void* stream)
{
    const int64_t npanels = (O + PANEL - 1) / PANEL;
    const int nsteps = (int)(Kpb / FRAG_KB);
    const int64_t nslots = npanels * nsteps * FRAGS_PER_PANEL * 64;
    const dim3 grid((unsigned)((nslots + 255) / 256)), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (elem_size(dtype) == 2)
        hipLaunchKernelGGL((k_decompose_packed<2, FUSED>), grid, block, 0, s, static_cast<const uint16_t*>(Wq), O, (int)K, N, true,
                           static_cast<uint4*>(w_vals), static_cast<uint32_t*>(w_meta), nslots, nsteps, violations);
    else
        hipLaunchKernelGGL((k_decompose_packed<1, FUSED>), grid, block, 0, s, static_cast<const uint8_t*>(Wq), O, (int)K, N, dtype == SS_FP8_E4M3,
                           static_cast<uint4*>(w_vals), static_cast<uint32_t*>(w_meta), nslots, nsteps, violations);
    return launch_status();
}

extern "C" ss_status slide_decompose(const void* Wq, int64_t O, int64_t K, int N, ss_dtype dtype, void* w_vals, void* w_meta,
                                     int32_t* violations, void* stream)
{
    ss_status st = check_decompose(O, K, N, dtype);
    if (st != SS_OK) return st;
    const int64_t Kpb = lifted_ld(K, N, elem_size(dtype)) * elem_size(dtype);
    if (O == 0) return SS_OK;
    if (!Wq || !w_vals || !w_meta) return SS_ERR_NULL;
    return launch_packed<false>(Wq, O, K, N, dtype, Kpb, w_vals, w_meta, violations, stream);
}

// Fused order: lifted bytes per row = 192 per 128 unlifted bytes (whole super-units; columns at and beyond K are zero).
static int64_t fused_lifted_row_bytes(int64_t K, ss_dtype dtype) { return (K * elem_size(dtype) + KSTEP - 1) / KSTEP * (3 * FRAG_KB); }

extern "C" ss_status slide_packed_sizes_fused(int64_t O, int64_t K, int N, ss_dtype dtype, size_t* vals_bytes, size_t* meta_bytes)
{
    ss_status st = check_decompose(O, K, N, dtype);
    if (st != SS_OK) return st;
    if (N != 4) return SS_ERR_BAD_PATTERN_N;
    if (!vals_bytes || !meta_bytes) return SS_ERR_NULL;
    const int64_t Kpb = fused_lifted_row_bytes(K, dtype);
    const int64_t Opad = (O + PANEL - 1) / PANEL * PANEL;
    *vals_bytes = (size_t)(Opad * (Kpb / 2));
    *meta_bytes = (size_t)(Opad * (Kpb / 8));
    return SS_OK;
}

extern "C" ss_status slide_decompose_fused(const void* Wq, int64_t O, int64_t K, int N, ss_dtype dtype, void* w_vals, void* w_meta,
                                           int32_t* violations, void* stream)
{
    ss_status st = check_decompose(O, K, N, dtype);
    if (st != SS_OK) return st;
    if (N != 4) return SS_ERR_BAD_PATTERN_N;
    if (O == 0) return SS_OK;
    if (!Wq || !w_vals || !w_meta) return SS_ERR_NULL;
    return launch_packed<true>(Wq, O, K, N, dtype, fused_lifted_row_bytes(K, dtype), w_vals, w_meta, violations, stream);
}

extern "C" ss_status slide_decompose_canonical(const void* Wq, int64_t O, int64_t K, int N, ss_dtype dtype, void* vals, uint8_t* idx,
                                               int32_t* violations, void* stream)
{
    ss_status st = check_decompose(O, K, N, dtype);
    if (st != SS_OK) return st;
    if (O == 0) return SS_OK;
    if (!Wq || !vals || !idx) return SS_ERR_NULL;
    const int64_t nwin = n_groups(K, N) * (N - 1);
    const int64_t total = O * nwin;
    dim3 grid((unsigned)((total + 255) / 256)), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (elem_size(dtype) == 2)
        hipLaunchKernelGGL(k_decompose_canonical<2>, grid, block, 0, s, static_cast<const uint16_t*>(Wq), O, (int)K, N, true,
                           static_cast<uint16_t*>(vals), idx, violations);
    else
        hipLaunchKernelGGL(k_decompose_canonical<1>, grid, block, 0, s, static_cast<const uint8_t*>(Wq), O, (int)K, N,
                           dtype == SS_FP8_E4M3, static_cast<uint8_t*>(vals), idx, violations);
    return launch_status();
}
