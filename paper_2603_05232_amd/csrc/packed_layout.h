// The opaque packed weight layout shared by slide_decompose (writer) and slide_sparse_gemm
// (reader).  It is ordered for the CDNA4 sparse matrix instructions so that one wavefront-wide
// 16-byte load fills the sparse-operand registers of one instruction and one 4-byte load fills
// its index register.  Everything is laid out in bytes of the lifted row: a "step" is 64 lifted
// bytes (64 columns of an 8-bit type, 32 of bf16), the depth of one sparse matrix instruction.
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
// bf16 uses v_smfmac_f32_32x32x32_bf16 (8 stored values + 16 index bits per lane, same bit
// positions [2p+1:2p]); measured: stored value p meets B element j = 8 qa + 4 ((p & 3) >> 1) + t
// of B lane (n, qb = p >> 2).  With B lane (n, qb) holding the 16 lifted columns
// [16 qb, 16 qb + 16) of the 32-column step, value p belongs to window
//     wi = 4 (w >> 1) + 2 qa + (w & 1),  w = p >> 1          (8 windows per step).
// The accumulator D[i][n] lives in lane n + 32 ((i >> 2) & 1), register (i & 3) + 4 (i >> 3).
//
// Output channels are grouped in panels of 128 = 4 fragments x 32 rows, and row i of fragment
// f is output channel  panel*128 + 64 ((i >> 2) & 1) + 16 f + 4 (i >> 3) + (i & 3),  which
// makes the 4 x 16 accumulator registers of a lane 64 consecutive output channels.
#pragma once
#include <stdint.h>

namespace ss {

constexpr int FRAG_ROWS = 32;       // rows of one sparse fragment
constexpr int FRAG_KB = 64;         // lifted bytes (per row) of one sparse fragment = one step
constexpr int FRAGS_PER_PANEL = 4;

// output-channel offset inside a 128-row panel of row i (0..31) of fragment f (0..3)
__host__ __device__ inline int panel_row(int f, int i) { return 64 * ((i >> 2) & 1) + 16 * f + 4 * (i >> 3) + (i & 3); }
// window inside a step held by lane half qa at window slot w of the lane; a lane holds HW = 4 / ES
// windows of each half of the step (ES = bytes per element: 8 slots of 16 windows, or 4 of 8)
template <int ES> __host__ __device__ inline int step_window(int qa, int w)
{
    constexpr int HW = 4 / ES;
    return 2 * HW * (w / HW) + HW * qa + (w % HW);
}

// Fused order of the 6:8 pattern (N = 4), for the GEMM that takes unlifted activations and applies the lifting
// operator on the way from LDS to the operand registers.  A super-unit is 128 unlifted bytes of a row = BL = 8 / ES
// blocks per B-lane half = three steps.  B lane (n, qb) holds the 64 unlifted bytes [64 qb, 64 qb + 64) of the
// super-unit as 16 registers; steps 3s and 3s+1 use registers 0..7 and 8..15 as they are (windows l = 0 and l = 2
// of a block are its first and second half: no data movement), step 3s+2 uses the middle windows (l = 1) of all
// the lane's blocks, built with one byte-align (8-bit types) or two register copies (16-bit types) per window.
// So window slot wsl (0..BL-1) of B lane half qb in step 3s+J is
//     J = 0, 1:  block (2s + qb) BL + J BL/2 + (wsl >> 1),  window l = 2 (wsl & 1)
//     J = 2:     block (2s + qb) BL + wsl,                  window l = 1
// and the A lane (qa, slot w) meets B lane half qb = w / HW, window slot wsl = HW qa + (w % HW) as in step_window.
template <int ES> __host__ __device__ inline void fused_window(int step, int qa, int w, int& g, int& l)
{
    constexpr int HW = 4 / ES, BL = 8 / ES;
    const int qb = w / HW, wsl = HW * qa + (w % HW);
    const int s = step / 3, J = step - 3 * s;
    l = J == 2 ? 1 : 2 * (wsl & 1);
    g = (2 * s + qb) * BL + (J == 2 ? wsl : J * (BL / 2) + (wsl >> 1));
}

// slot of the 16-byte value group of (panel, step, fragment, lane); values are stored [panel][step][fragment][lane],
// index words (4 bytes each, the upper half unused for bf16) [panel][step][lane][fragment], so that one 16-byte
// read hands a lane the words of all four fragments
__host__ __device__ inline int64_t frag_slot(int64_t panel, int64_t nsteps, int64_t step, int f, int lane)
{
    return ((panel * nsteps + step) * FRAGS_PER_PANEL + f) * 64 + lane;
}

}  // namespace ss
