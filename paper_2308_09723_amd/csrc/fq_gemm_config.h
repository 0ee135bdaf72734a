// Compile-time configuration shared by the host-side plan and the kernel dispatch.
#ifndef FQ_GEMM_CONFIG_H_
#define FQ_GEMM_CONFIG_H_

namespace fqd {

constexpr int MMA_NT = 3;       // column tiles per wave of the large-M kernel

// Ring depth (k-blocks in flight) of the pipelined form of the large-M kernel for the 64-row and
// the 32-row block shapes; 0 selects the two-buffer form.  The 128-row, 8-wave shape uses depth 2.
// Measured on the OPT-175B shapes at M = 32 and 64: depth 2 is 2-6 % faster than the two-buffer form,
// depths 3 and 4 are slower (their registers cost a resident wave per SIMD).
constexpr int FQ_RING_MT4 = 2;
constexpr int FQ_RING_MT2 = 2;

// Post-scaled form of the large-M kernel (codes converted without their scale, one fold per scale
// group and output tile): used where the conversion, not the matrix pipe, sets the pace, i.e. 3- and
// 4-bit codes and at most 64 rows per block.  Measured on the OPT-175B shapes (M = 32 / 64, us, pre- ->
// post-scaled): bf16 needs 23 vector instructions per 8 weights pre-scaled and 7 post-scaled (no packed
// bf16 arithmetic), QKV M=32 63 -> 52, FC1 89 -> 68, and at 64 rows with one scale row per k-block FC1
// 112 -> 100; with two scale rows per k-block the folds eat the gain at 64 rows (93 -> 127) but not at
// 32 (65 -> 62).  fp16 (13 -> 9 instructions) gains with one scale row only: FC1 M=32 74 -> 66, M=64
// 100 -> 94; with two it loses (54 -> 60).  8-bit codes gain nothing (M=32) or lose (M=64: 114 -> 127).
constexpr bool use_post(int act, int bits, int mt, int sr, int pipe) {
    if (pipe == 0 || bits == 8) return false;
    if (act == 0) return sr == 1 && mt <= 4;
    return (mt <= 2 && sr <= 2) || (mt == 4 && sr == 1);
}

// Small-M kernel variants that are compiled in: (NT column tiles per wave, ring DEPTH,
// register class = maximum waves per block).  The plan picks one of them plus the run-time
// block shape (GP column groups x KW k-workers).
//   variant 0: NT 3, DEPTH 2, up to 12 waves     variant 1: NT 3, DEPTH 3, up to 8 waves
//   variant 2: NT 1, DEPTH 4, up to 12 waves     variant 3: NT 2, DEPTH 3, up to 12 waves
struct SkinnyVariant { int nt, depth, maxw; };
constexpr SkinnyVariant SKINNY_VARIANTS[4] = {{3, 2, 12}, {3, 3, 8}, {1, 4, 12}, {2, 3, 12}};


}  // namespace fqd

#endif  // FQ_GEMM_CONFIG_H_
