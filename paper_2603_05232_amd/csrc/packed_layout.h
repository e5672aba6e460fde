// The opaque packed weight layout shared by slide_decompose (writer) and slide_sparse_gemm
// (reader).  It is ordered for the CDNA4 sparse matrix instructions so that one wavefront-wide
// 16-byte load fills the sparse-operand registers of one instruction and one 4-byte load fills
// its index register.
//
// 8-bit types use v_smfmac_*_32x32x64 (sparse operand A = 32 output channels x 64 lifted
// columns, 16 stored values + 32 index bits per lane).  Measured operand semantics of that
// instruction on gfx950: lane L holds A row i = L % 32, lane half qa = L / 32; its stored value
// p (byte p of the four A registers, p = 0..15) with 2-bit index t taken from bits [2p+1:2p] of
// the index register multiplies B element j = 16 qa + 4 ((p & 7) >> 1) + t of the B lane
// (n, qb = p >> 3), where B lane L' holds column n = L' % 32 and half qb = L' / 32.  The GEMM
// gives B lane (n, qb) the 32 lifted columns [32 qb, 32 qb + 32) of token n within the
// 64-column step, so stored value p of A lane (i, qa) belongs to window
//     wi = 8 (w >> 2) + 4 qa + (w & 3),  w = p >> 1          (16 windows per step).
// The accumulator D[i][n] lives in lane n + 32 ((i >> 2) & 1), register (i & 3) + 4 (i >> 3).
//
// Output channels are grouped in panels of 128 = 4 fragments x 32 rows, and row i of fragment
// f is output channel  panel*128 + 64 ((i >> 2) & 1) + 16 f + 4 (i >> 3) + (i & 3),  which
// makes the 4 x 16 accumulator registers of a lane 64 consecutive output channels.
#pragma once
#include <stdint.h>

namespace ss {

constexpr int FRAG_ROWS = 32;       // rows of one sparse fragment
constexpr int FRAG_K8 = 64;         // lifted columns of one 8-bit sparse fragment
constexpr int FRAGS_PER_PANEL = 4;

// output-channel offset inside a 128-row panel of row i (0..31) of fragment f (0..3)
__host__ __device__ inline int panel_row(int f, int i) { return 64 * ((i >> 2) & 1) + 16 * f + 4 * (i >> 3) + (i & 3); }
// window (0..15) inside a 64-column step held by lane half qa at window slot w (0..7)
__host__ __device__ inline int step_window(int qa, int w) { return 8 * (w >> 2) + 4 * qa + (w & 3); }

// slot of the 16-byte value group of (panel, step, fragment, lane); values are stored [panel][step][fragment][lane],
// index words [panel][step][lane][fragment] so that one 16-byte read hands a lane the words of all four fragments
__host__ __device__ inline int64_t frag_slot(int64_t panel, int64_t nsteps, int64_t step, int f, int lane)
{
    return ((panel * nsteps + step) * FRAGS_PER_PANEL + f) * 64 + lane;
}

}  // namespace ss
