// Compile-time configuration shared by the host-side plan and the kernel dispatch.
#ifndef FQ_GEMM_CONFIG_H_
#define FQ_GEMM_CONFIG_H_

namespace fqd {

constexpr int MMA_NT = 3;       // column tiles per wave of the large-M kernel

// Ring depth (k-blocks in flight) of the pipelined form of the large-M kernel for the 64-row and
// the 32-row block shapes; 0 selects the two-buffer form.  The 128-row, 8-wave shape uses depth 2.
// Measured on the OPT-175B shapes at M = 32 and 64: depth 2 is 2-6 % faster than the two-buffer form,
// depths 3 and 4 are slower (their registers cost a resident wave per SIMD).
#ifndef FQ_RING_MT4
#define FQ_RING_MT4 2
#endif
#ifndef FQ_RING_MT2
#define FQ_RING_MT2 2
#endif

// Small-M kernel variants that are compiled in: (NT column tiles per wave, ring DEPTH,
// register class = maximum waves per block).  The plan picks one of them plus the run-time
// block shape (GP column groups x KW k-workers).
//   variant 0: NT 3, DEPTH 2, up to 12 waves     variant 1: NT 3, DEPTH 3, up to 8 waves
//   variant 2: NT 1, DEPTH 4, up to 12 waves     variant 3: NT 2, DEPTH 3, up to 12 waves
struct SkinnyVariant { int nt, depth, maxw; };
constexpr SkinnyVariant SKINNY_VARIANTS[4] = {{3, 2, 12}, {3, 3, 8}, {1, 4, 12}, {2, 3, 12}};


}  // namespace fqd

#endif  // FQ_GEMM_CONFIG_H_
