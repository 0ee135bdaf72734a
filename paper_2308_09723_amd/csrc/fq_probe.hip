// Measurement helper, not part of the method: what rate do this GPU's matrix pipes hold on the caller's
// operand values?  The chip's clock under load follows the switching activity of the operands, so the
// vendor's peak (quoted at the nominal clock) is reached on all-zero operands only; on random ones a
// loop of nothing but MFMAs runs well below it.  The tiled product kernel is compared with this next
// to the vendor's peak.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "fq_internal.h"

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int PROBE_BLOCKS = 1024;      // four rounds of one 8-wave block per compute unit
constexpr int PROBE_TILE_UNITS = 2048;  // 32 KiB of activation-like operands per block, in 16-byte units
constexpr int PROBE_TILES = 64;

// The loop of the 128-row block shape of the tiled product without its loads, conversions and barrier: per
// iteration and wave 4 k-steps x 8 row tiles x 3 column tiles of v_mfma_f32_16x16x32_f16; LDS: one 16-byte
// fragment read per lane and three MFMAs (as in the product), or none.  INT8: the same loop with
// v_mfma_i32_16x16x64_i8 (the integer path's instruction: twice the operations per MFMA).
template <bool LDS_READS, bool INT8>
__global__ __launch_bounds__(512) void fq_mfma_rate_kernel(const u32x4* __restrict__ operands,
                                                           float* __restrict__ sink, int iterations) {
    extern __shared__ u32x4 lds[];   // [PROBE_TILE_UNITS]
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i < PROBE_TILE_UNITS; i += 512)
        lds[i] = operands[(blockIdx.x % PROBE_TILES) * PROBE_TILE_UNITS + i];
    __syncthreads();
    u32x4 w[3];
#pragma unroll
    for (int n = 0; n < 3; ++n) w[n] = operands[PROBE_TILES * PROBE_TILE_UNITS + tid * 3 + n];
    typedef typename std::conditional<INT8, v4i, f32x4>::type ACC;
    ACC acc[8][3];
    u32x4 a[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) {
        a[m] = lds[(m * 256 + lane) % PROBE_TILE_UNITS];
#pragma unroll
        for (int n = 0; n < 3; ++n) acc[m][n] = ACC{0, 0, 0, 0};
    }
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                if constexpr (LDS_READS) a[m] = lds[((it * 4 + t) * 64 + m * 256 + lane) % PROBE_TILE_UNITS];
#pragma unroll
                for (int n = 0; n < 3; ++n) {
                    if constexpr (INT8)
                        acc[m][n] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, w[n]),
                                                                          __builtin_bit_cast(v4i, a[m]), acc[m][n], 0, 0, 0);
                    else
                        acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, w[n]),
                                                                           __builtin_bit_cast(f16x8, a[m]), acc[m][n], 0, 0, 0);
                }
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int m = 0; m < 8; ++m)
#pragma unroll
        for (int n = 0; n < 3; ++n) s += (float)acc[m][n][0] + (float)acc[m][n][1] + (float)acc[m][n][2] + (float)acc[m][n][3];
    sink[blockIdx.x * 512 + tid] = s;
}

}  // namespace

size_t fq_mfma_probe_operand_bytes() { return ((size_t)PROBE_TILES * PROBE_TILE_UNITS + 512 * 3) * 16; }
size_t fq_mfma_probe_sink_bytes() { return (size_t)PROBE_BLOCKS * 512 * sizeof(float); }
double fq_mfma_probe_flops(int iterations, int int8) {
    return (double)PROBE_BLOCKS * 8.0 * (double)iterations * 96.0 * (2.0 * 16 * 16 * (int8 ? 64 : 32));
}

int fq_launch_mfma_rate_probe(const void* operands, void* sink, int iterations, int lds_reads, int int8,
                              hipStream_t stream) {
#define FQ_PROBE_GO(L_, I_)                                                                                    \
    hipLaunchKernelGGL((fq_mfma_rate_kernel<L_, I_>), dim3(PROBE_BLOCKS), dim3(512), PROBE_TILE_UNITS * 16, stream, \
                       (const u32x4*)operands, (float*)sink, iterations)
    if (int8) {
        if (lds_reads) FQ_PROBE_GO(true, true);
        else FQ_PROBE_GO(false, true);
    } else {
        if (lds_reads) FQ_PROBE_GO(true, false);
        else FQ_PROBE_GO(false, false);
    }
#undef FQ_PROBE_GO
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}
