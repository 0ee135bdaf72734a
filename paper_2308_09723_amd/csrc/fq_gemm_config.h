// Compile-time configuration shared by the host-side plan and the kernel dispatch.
#ifndef FQ_GEMM_CONFIG_H_
#define FQ_GEMM_CONFIG_H_

namespace fqd {

constexpr int MMA_NT = 3;       // column tiles per wave of the large-M kernel

// Small-M kernel variants that are compiled in: (NT column tiles per wave, ring DEPTH,
// register class = maximum waves per block).  The plan picks one of them plus the run-time
// block shape (GP column groups x KW k-workers).
//   variant 0: NT 3, DEPTH 2, up to 12 waves     variant 1: NT 3, DEPTH 3, up to 8 waves
//   variant 2: NT 1, DEPTH 4, up to 12 waves     variant 3: NT 2, DEPTH 3, up to 12 waves
struct SkinnyVariant { int nt, depth, maxw; };
constexpr SkinnyVariant SKINNY_VARIANTS[4] = {{3, 2, 12}, {3, 3, 8}, {1, 4, 12}, {2, 3, 12}};


}  // namespace fqd

#endif  // FQ_GEMM_CONFIG_H_
