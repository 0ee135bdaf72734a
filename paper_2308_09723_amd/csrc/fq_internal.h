// Internal launcher declarations shared by the translation units of libfq.
#ifndef FQ_INTERNAL_H_
#define FQ_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/fq.h"

// quantiser side (sfmt: an fq_scale_format)
int fq_launch_quantize(const void* W, int64_t K, int64_t N, int bits, int g, int sfmt, void* codes, void* scales,
                       hipStream_t stream);
int fq_launch_unpack(const void* codes, int64_t K, int64_t N, int bits, int8_t* q, hipStream_t stream);
int64_t fq_quant_error_blocks(int64_t K, int64_t N);
int fq_launch_quant_error(const void* W, int64_t K, int64_t N, int bits, int g, int sfmt, const void* codes,
                          const void* scales, double* out_host2, void* workspace, hipStream_t stream);
int fq_launch_choose_group(const void* W, int64_t K, int64_t N, int g_top, int levels, float alpha,
                           int* flags_host, void* workspace, hipStream_t stream);

// measurement helper: a kernel that only reads a buffer
int fq_launch_stream_read_probe(const void* buf, size_t bytes, void* sink, hipStream_t stream);
size_t fq_mfma_probe_operand_bytes();
size_t fq_mfma_probe_sink_bytes();
double fq_mfma_probe_flops(int iterations, int int8);
int fq_launch_mfma_rate_probe(const void* operands, void* sink, int iterations, int lds_reads, int int8,
                              hipStream_t stream);

// product side
struct fq_gemm_plan {
    int kind;      // 0 = skinny (M <= 16), 1 = tiled
    int mt;        // row tiles of 16 per block (tiled kernel)
    int waves;     // waves per block
    int variant;   // small-M kernel: which compiled variant (NT, ring depth, register class)
    int gp, kw;    // small-M kernel: column groups x k-workers per block
    int au;        // small-M kernel: activation units a lane stages per super-block (1, 2 or 4)
    int splits;    // split-K factor (>= 1)
    int kb_per_split;   // k-blocks per grid split (tiled) or per wave (small-M)
    // tiled kernel, splits == 1 only: the last `tail_tiles` output tiles (the partly filled last round
    // of blocks) are split `tail_splits` ways along K so that they fill the idle compute units
    int tail_tiles, tail_splits, tail_kbs;
};
fq_gemm_plan fq_plan_gemm(int64_t M, int64_t N, int64_t K, int bits, int g);
// compute units of the device (asked once per process; 256 without a device)
int fq_cu_count();
// Rows of K per k-block of the tiled kernel for a block shape (the unit of kb_per_split and tail_kbs):
// the layout's k-block, except that the 128-row, 8-wave shape takes two 64-row blocks of 8-bit codes at a
// time when K allows it and such a k-block lies inside one scale group (with two scale rows the wider
// kernel spills and gains nothing, with four it loses).
inline int fq_mma_kblk(int bits, int mt, int waves, int64_t K, int g) {
    return (bits == 8 && mt == 8 && waves == 8 && K % 128 == 0 && g % 128 == 0) ? 128 : (bits == 8 ? 64 : 128);
}
// Workspace layout of fq_gemm: [split-K partial tiles][bf16 activations rewritten as binary16][their M row scales,
// then 2^-E and 2^E of the scale matrix (bfloat16 scales), then FQ_SCALE_PARTS words of the search for E]
inline size_t fq_partial_bytes(const fq_gemm_plan& p, int64_t M, int64_t N) {
    const int parts = p.splits > 1 ? p.splits : (p.tail_tiles > 0 ? p.tail_splits : 0);
    return (size_t)parts * (size_t)M * (size_t)N * sizeof(float);
}
inline size_t fq_a16_bytes(int64_t M, int64_t K) { return (((size_t)M * (size_t)K * 2) + 255) / 256 * 256; }
#define FQ_SCALE_PARTS 256
inline size_t fq_rowscale_bytes(int64_t M) { return ((size_t)M + 2 + FQ_SCALE_PARTS) * sizeof(float); }
// bf16 activations (binary16 or bfloat16 scales) take the fp16 matrix path for the 128-row shapes of wide
// matrices: the rewrite of the rows costs 4 M K bytes of traffic against 2 M N K flops
inline bool fq_via_f16(int act_dtype, int scale_format, const fq_gemm_plan& p, int64_t N) {
    (void)scale_format;
    return act_dtype == FQ_BF16 && p.kind == 1 && p.mt == 8 && N >= 8192;
}
// act: FQ_F16, FQ_BF16, or 2 = bf16 activations with bf16 scales
int fq_launch_gemm(const void* A, int act, int64_t M, int64_t N, int64_t K, const void* codes,
                   const void* scales, int bits, int g, void* C, void* workspace, hipStream_t stream);
int fq_launch_gemm_grouped(const void* A, int act, const int32_t* offsets, int E, int64_t N, int64_t K,
                           const void* codes, const void* scales, int bits, int g, void* C,
                           hipStream_t stream);

#endif  // FQ_INTERNAL_H_
