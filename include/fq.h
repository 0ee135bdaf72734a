/*
 * fq.h -- C ABI of the fine-grained weight-only quantisation library for MI355X (gfx950).
 *
 * The library implements the hot path of "FineQuant: Unlocking Efficiency with
 * Fine-Grained Weight-Only Quantization for LLMs": a linear abs-max symmetric
 * quantiser with one half-precision scale per block of g consecutive rows of a
 * column, and the fused dequantise-and-multiply product C = A . dequant(W).
 *
 * Conventions (all entry points):
 *   - plain C, no exceptions; every int-returning call returns an fq_status.
 *   - every buffer is CALLER-OWNED DEVICE memory unless the comment says "host";
 *     the library neither allocates, frees nor retains any of them.
 *   - matrices are row-major; the weight matrix is W[K, N] so that y = x . W and
 *     a "column" is an output channel (section 4.1, "Quantization Method").
 *   - device pointers must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls are asynchronous on that stream unless stated otherwise.
 *   - arguments are validated on the host before anything is launched, so
 *     invalid calls never touch the GPU.
 */
#ifndef FQ_H_
#define FQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fq_status {
    FQ_OK = 0,
    FQ_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad enum, group size not dividing K */
    FQ_ERR_UNSUPPORTED = 2, /* valid in principle, but outside what the kernels handle (see each call) */
    FQ_ERR_WORKSPACE = 3,   /* workspace missing or smaller than fq_gemm_workspace_bytes() */
    FQ_ERR_HIP = 4          /* a HIP runtime call failed (launch error, wrong device, ...) */
} fq_status;

typedef enum fq_dtype {
    FQ_F16 = 0, /* IEEE binary16 activations and output */
    FQ_BF16 = 1 /* bfloat16 activations and output */
} fq_dtype;

/* Storage format of the scale matrix.  Appendix B stores the scales in half precision; the
 * kernels of section 4.1 ("GPU kernel implementations") take scales of the activation's data
 * type, i.e. bfloat16 scales next to bfloat16 activations.  The entry points without a
 * `scale_format` argument use FQ_SCALE_F16 (for either activation type); the *_sf entry points
 * take the format explicitly.  FQ_SCALE_BF16 changes the encoding: the quantiser then picks the
 * smallest BFLOAT16 s with (2^bits - 1) * s >= 2 max|w| and divides by that s. */
typedef enum fq_scale_format {
    FQ_SCALE_F16 = 0, /* IEEE binary16 scales */
    FQ_SCALE_BF16 = 1 /* bfloat16 scales; products accept them with FQ_BF16 activations only */
} fq_scale_format;

/* Shape limits shared by every call:
 *   bits        3, 4 or 8 (3-bit codes: the paper evaluates them for accuracy, section 4.2 and
 *               Table 5, whose int3 footprints are 3 + 16/g bits per weight)
 *   N           multiple of 16
 *   K           multiple of 128 (bits = 3, 4) or 64 (bits = 8)
 *   group_size  0 or K (one scale per column), or a multiple of 32 that divides K
 *               (section 5 plans kernels for every power-of-two group size
 *               above 16; multiples of 32 cover that from 32 up).
 */

/* Size in bytes of the packed code buffer: K*N*bits/8 (no padding).  0 on invalid arguments. */
size_t fq_codes_bytes(int64_t K, int64_t N, int bits);

/* Size in bytes of the scale matrix [K/g, N] of 16-bit values (either format).  0 on invalid arguments. */
size_t fq_scales_bytes(int64_t K, int64_t N, int group_size);

/* Bytes of scratch fq_gemm needs for this problem (split-K partial sums, rewritten activations; may be
 * 0).  The value is an upper bound that depends only on the arguments. */
size_t fq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int bits, int group_size);

/* The exact need of fq_gemm / fq_gemm_sf for one activation type (an fq_dtype) and scale format (an
 * fq_scale_format); fq_gemm_workspace_bytes() is the largest of these.  (bfloat16 activations of wide
 * matrices are rewritten row by row before the product, which takes M*K*2 + M*4 bytes more.) */
size_t fq_gemm_workspace_bytes_for(int64_t M, int64_t N, int64_t K, int bits, int group_size, int act_dtype,
                                   int scale_format);

/* Same for fq_gemm_grouped, with total_rows = offsets[E]. */
size_t fq_gemm_grouped_workspace_bytes(int64_t total_rows, int E, int64_t N, int64_t K, int bits,
                                       int group_size);

/*
 * fq_quantize -- Appendix A ("Linear quantization with absolute maximum") applied per
 * block of `group_size` consecutive rows of each column (section 4.1, "Quantization
 * Method"), scales stored in half precision (Appendix B).
 *
 *   m = max |w| over the block;  s = smallest binary16 value with (2^bits - 1) * s >= 2 m;
 *   q = clamp(round_half_even(w / s), -(2^(bits-1) - 1), +(2^(bits-1) - 1)), the quotient
 *   taken in IEEE binary32;  an all-zero block gives s = 0, q = 0.
 *
 *   W_f16      in   [K, N] binary16, row-major, finite values
 *   codes      out  fq_codes_bytes() bytes; opaque tiled layout consumed by fq_gemm / fq_unpack
 *   scales_f16 out  [K/g, N] binary16, row-major
 * Errors: FQ_ERR_INVALID_ARG (null pointers, bad bits, g not dividing K),
 *         FQ_ERR_UNSUPPORTED (shape limits above), FQ_ERR_HIP.
 */
int fq_quantize(const void* W_f16, int64_t K, int64_t N, int bits, int group_size, void* codes,
                void* scales_f16, void* stream);

/* fq_quantize with the scale matrix stored as `scale_format` (an fq_scale_format); `scales` is
 * [K/g, N] 16-bit values of that format.  fq_quantize(...) = fq_quantize_sf(..., FQ_SCALE_F16, ...).
 * Errors: as fq_quantize; FQ_ERR_INVALID_ARG for an unknown format. */
int fq_quantize_sf(const void* W_f16, int64_t K, int64_t N, int bits, int group_size, int scale_format,
                   void* codes, void* scales, void* stream);

/*
 * fq_unpack -- inverse of the packing step: writes the logical signed codes q[K, N]
 * (int8, row-major) held in a packed buffer.  Used for parity checks and debugging.
 */
int fq_unpack(const void* codes, int64_t K, int64_t N, int bits, int8_t* q, void* stream);

/*
 * fq_choose_group -- the adaptive fine-grained heuristic of section 3.3: start from
 * g_start (0 = one group per column), and while the halved size is an integer >= g_min,
 * halve it if for ANY group the smaller abs-max of its two halves is below
 * (1 - alpha) times the group's abs-max (comparison in binary32); stop at the first
 * size for which no group changes that much.  One group size per matrix.
 *
 *   g_out  out  HOST pointer; receives the chosen group size.
 * The call enqueues its kernels on `stream`, then SYNCHRONISES that stream to read
 * the result back.  `workspace` is device scratch of at least
 * fq_choose_group_workspace_bytes(K, N, g_start, g_min) bytes.
 * The returned size is not checked against fq_gemm's limits (it may be odd multiples
 * of small numbers when K has odd factors); callers pass g_start / g_min accordingly.
 * Errors: FQ_ERR_INVALID_ARG (null pointers, alpha outside [0, 1], g_start not dividing K),
 *         FQ_ERR_UNSUPPORTED (N not a multiple of 16, more than 24 halvings, more than 65535
 *         groups per column), FQ_ERR_WORKSPACE, FQ_ERR_HIP.
 */
size_t fq_choose_group_workspace_bytes(int64_t K, int64_t N, int g_start, int g_min);
int fq_choose_group(const void* W_f16, int64_t K, int64_t N, int g_start, int g_min, float alpha,
                    int* g_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * fq_quant_error -- the quantisation error that section 3.2 studies as a function of the
 * group size (figure 2a: mean squared error between a weight matrix and its dequantised
 * codes, the dequantised value being q * s as in Appendix A):
 *   sse = sum over all (k, n) of (W[k, n] - q[k, n] * s[k / g, n])^2,   max_abs = max |...|,
 * evaluated in binary64 (every difference is exact; only the additions round) in a fixed
 * order, so the result is deterministic.  The mean squared error is sse / (K * N).
 *
 *   W_f16, codes, scales_f16  in   as given to / written by fq_quantize for (K, N, bits, group_size)
 *   sse_out, max_abs_out      out  HOST pointers
 *   workspace                      device scratch, >= fq_quant_error_workspace_bytes(K, N) bytes
 * The call enqueues its kernels on `stream`, then SYNCHRONISES that stream to read the two
 * numbers back.  Errors: as fq_quantize, plus FQ_ERR_WORKSPACE.
 */
size_t fq_quant_error_workspace_bytes(int64_t K, int64_t N);
int fq_quant_error(const void* W_f16, int64_t K, int64_t N, int bits, int group_size, const void* codes,
                   const void* scales_f16, double* sse_out, double* max_abs_out, void* workspace,
                   size_t workspace_bytes, void* stream);

/* fq_quant_error for scales stored as `scale_format`. */
int fq_quant_error_sf(const void* W_f16, int64_t K, int64_t N, int bits, int group_size, int scale_format,
                      const void* codes, const void* scales, double* sse_out, double* max_abs_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * fq_gemm -- the fused dequantise-and-multiply product of section 4.1 ("GPU kernel
 * implementations"):  C[m, n] = sum_k A[m, k] * (q[k, n] * s[k / g, n]),
 * accumulated in binary32, written in the activation's data type.  (For bfloat16 activations and
 * wide matrices with many rows the product is evaluated on the fp16 matrix path after each
 * activation row has been divided by a power of two that fits it into binary16; the result is
 * rescaled exactly and rounded to bfloat16 once; every bfloat16 magnitude has such a power of two, so rows
 * of any size keep their relative precision.  With bfloat16 scales the scale matrix is likewise
 * divided by the power of two of its largest scale, and scales more than 2^14 times smaller than that one lose
 * low bits or vanish.)
 *
 *   A           in   [M, K] row-major, act_dtype
 *   codes       in   packed codes written by fq_quantize for the same (K, N, bits)
 *   scales_f16  in   [K/g, N] binary16
 *   C           out  [M, N] row-major, act_dtype
 *   workspace        device scratch, >= fq_gemm_workspace_bytes(M, N, K, bits, group_size)
 *                    bytes (may be NULL when that is 0)
 * M = 0 is a valid no-op.  Deterministic: the same inputs give the same bits.
 * The call only enqueues kernels on `stream` (no allocation, no memset, no synchronisation), so it
 * may be recorded into a HIP graph by stream capture once every kernel shape involved has been
 * launched normally before (the first launch of some shapes raises their LDS limit, which is a
 * host-side call).  Calls that share a workspace must be ordered on one stream.
 * Errors: as fq_quantize, plus FQ_ERR_WORKSPACE.
 */
int fq_gemm(const void* A, int act_dtype, int64_t M, int64_t N, int64_t K, const void* codes,
            const void* scales_f16, int bits, int group_size, void* C, void* workspace,
            size_t workspace_bytes, void* stream);

/* fq_gemm with the scale matrix stored as `scale_format`, written by fq_quantize_sf with the same
 * format (section 4.1: scales of the activation's data type).  FQ_SCALE_BF16 requires
 * act_dtype = FQ_BF16 (otherwise FQ_ERR_UNSUPPORTED); FQ_SCALE_F16 is fq_gemm itself. */
int fq_gemm_sf(const void* A, int act_dtype, int64_t M, int64_t N, int64_t K, const void* codes,
               const void* scales, int scale_format, int bits, int group_size, void* C, void* workspace,
               size_t workspace_bytes, void* stream);

/*
 * fq_gemm_noalloc -- fq_gemm for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch
 * fq_gemm takes as `workspace` (split-K partial sums, rewritten bfloat16 activation rows) lives in a
 * device array that is part of the library's code object: FQ_NOALLOC_SCRATCH_BYTES bytes on every GPU
 * the library runs on, held until the process ends.  The call allocates and frees nothing and runs the
 * same kernels as fq_gemm (binary16 scales), so the results are bit-identical to fq_gemm's.
 *
 *   arguments  as fq_gemm, without the workspace
 * Errors: as fq_gemm; FQ_ERR_WORKSPACE when the problem needs more scratch than the array holds
 *         (fq_gemm_workspace_bytes_for(...) > FQ_NOALLOC_SCRATCH_BYTES: nothing is launched; use fq_gemm).
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents (no kernel reads
 * what an earlier kernel of the same call has not written, so nothing needs clearing).  Calls that
 * overlap on one GPU (two streams, two host threads) RACE on it: order them on one stream.  The first
 * call on a device looks up the array's address (a host-side query); make one call outside any stream
 * capture before capturing.
 */
#define FQ_NOALLOC_SCRATCH_BYTES (64u << 20)
int fq_gemm_noalloc(const void* A, int act_dtype, int64_t M, int64_t N, int64_t K, const void* codes,
                    const void* scales_f16, int bits, int group_size, void* C, void* stream);
/* FQ_NOALLOC_SCRATCH_BYTES as the built library has it. */
size_t fq_gemm_noalloc_scratch_bytes(void);

/*
 * fq_gemm_grouped -- the same product for the expert FFNs of a mixture-of-experts
 * layer (section 4.3): rows offsets[e] .. offsets[e+1]-1 of A (tokens sorted by
 * expert) are multiplied by expert e's matrix.  Experts without rows are skipped
 * and their weights are not read.
 *
 *   offsets_host  in  HOST array [E+1], non-decreasing, offsets[0] = 0
 *   codes         in  E packed matrices back to back (fq_codes_bytes() apart)
 *   scales_f16    in  E scale matrices back to back (fq_scales_bytes() apart)
 *   A, C              [offsets[E], K] and [offsets[E], N]
 * E <= 256.
 * Experts are cut into row tiles of up to three sizes and each size is one kernel; these
 * independent kernels run on `stream` and on two streams the library creates (once per
 * device, default priority, never destroyed), forked from and joined back to `stream` with
 * events, so the call still behaves as one asynchronous operation on `stream`.  Calls from several host
 * threads are serialised on the host while they enqueue (the side streams and events are shared).
 */
int fq_gemm_grouped(const void* A, int act_dtype, const int32_t* offsets_host, int E, int64_t N,
                    int64_t K, const void* codes, const void* scales_f16, int bits, int group_size,
                    void* C, void* workspace, size_t workspace_bytes, void* stream);

/* fq_gemm_grouped with the scale matrices stored as `scale_format` (same rule as fq_gemm_sf). */
int fq_gemm_grouped_sf(const void* A, int act_dtype, const int32_t* offsets_host, int E, int64_t N,
                       int64_t K, const void* codes, const void* scales, int scale_format, int bits,
                       int group_size, void* C, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The integer path -- int8 activations x int4 weights with INTEGER group scales, multiplied on the integer
 * matrix cores.  Section 5 ("Conclusions and Limitations", last paragraph) names it as future work and gives
 * no formula; the reading implemented here keeps Appendix A's quantiser and section 4.1's groups:
 *   weights      s[i, n] = z[i, n] * t[n]: one binary16 step t per column (the smallest with
 *                16 * 15 * t >= 2 max|w| over the column) and one integer multiplier z in 1..16 per group (the
 *                smallest with 15 * z * t >= 2 max|w| over the group), one byte each;
 *                q = clamp(round_half_even(w / (z t)), -7, 7), binary32 quotient.  |q z t - w| <= z t / 2 holds
 *                exactly, and q * z is an int8 (at most 112 in magnitude).
 *   activations  Appendix A at 8 bits per row: alpha[m] = the smallest binary32 with 255 alpha >= 2 max|A[m, :]|,
 *                a = clamp(round_half_even(A / alpha), -127, 127), binary32 quotient.
 *   product      S[m, n] = sum_k a[m, k] * q[k, n] * z[k / g, n] in exact int32 arithmetic (K <= 131072 keeps
 *                |S| < 2^31),  C[m, n] = alpha[m] * t[n] * S[m, n] evaluated in binary32, rounded to out_dtype.
 * Shape limits: N a multiple of 16, K a multiple of 128 and at most 131072, group_size 0 / K or a multiple of 32
 * that divides K.  The packed codes take fq_codes_bytes(K, N, 4) bytes in a tiled layout of this path's own
 * (ordered for the 64-deep int8 MFMA; fq_unpack does NOT read it, fq_unpack_w4a8 does).
 */

/* Size in bytes of the multiplier matrix z[K/g, N] (one byte per group).  0 on invalid arguments. */
size_t fq_zscale_bytes(int64_t K, int64_t N, int group_size);

/*
 * fq_quantize_w4a8 -- the weight quantiser of the integer path.
 *   W_f16      in   [K, N] binary16, row-major, finite
 *   codes      out  fq_codes_bytes(K, N, 4) bytes (also used as scratch for the groups' abs-max on the way)
 *   zscale     out  [K/g, N] bytes, values 1..16
 *   tstep_f16  out  [N] binary16
 * Errors: FQ_ERR_INVALID_ARG, FQ_ERR_UNSUPPORTED (shape limits above), FQ_ERR_HIP.
 */
int fq_quantize_w4a8(const void* W_f16, int64_t K, int64_t N, int group_size, void* codes, uint8_t* zscale,
                     void* tstep_f16, void* stream);

/* fq_unpack_w4a8 -- the logical signed codes q[K, N] (int8, row-major) of a buffer written by fq_quantize_w4a8. */
int fq_unpack_w4a8(const void* codes, int64_t K, int64_t N, int8_t* q, void* stream);

/*
 * fq_quantize_act_i8 -- the activation quantiser of the integer path (one scale per row).
 *   A      in   [M, K] row-major, act_dtype (FQ_F16 or FQ_BF16), finite
 *   Aq     out  [M, K] int8, row-major
 *   alpha  out  [M] binary32
 * M = 0 is a valid no-op.  Errors: FQ_ERR_INVALID_ARG, FQ_ERR_UNSUPPORTED (M or K above 2^24), FQ_ERR_HIP.
 */
int fq_quantize_act_i8(const void* A, int act_dtype, int64_t M, int64_t K, int8_t* Aq, float* alpha, void* stream);

/*
 * fq_gemm_w4a8 -- the product of the integer path.
 *   Aq, alpha            in   as written by fq_quantize_act_i8
 *   codes, zscale, tstep in   as written by fq_quantize_w4a8 for the same (K, N, group_size)
 *   C                    out  [M, N] row-major, out_dtype (FQ_F16 or FQ_BF16)
 *   workspace                 device scratch, >= fq_gemm_w4a8_workspace_bytes(M, N, K, group_size) bytes (int32 sums
 *                             of products whose K range is split over several blocks; may be NULL when that is 0)
 * Asynchronous on `stream`, no allocation, deterministic.
 * M = 0 is a valid no-op.  Errors: FQ_ERR_INVALID_ARG, FQ_ERR_UNSUPPORTED, FQ_ERR_WORKSPACE, FQ_ERR_HIP.
 */
size_t fq_gemm_w4a8_workspace_bytes(int64_t M, int64_t N, int64_t K, int group_size);
int fq_gemm_w4a8(const int8_t* Aq, const float* alpha, int64_t M, int64_t N, int64_t K, const void* codes,
                 const uint8_t* zscale, const void* tstep_f16, int group_size, void* C, int out_dtype,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * fq_gemm_describe -- writes a short text description of the kernel configuration fq_gemm
 * would use for this problem (kernel family, tile shape, block shape, split-K factor) into
 * buf (HOST memory, at most buf_bytes including the terminating 0).  For logs and benchmark
 * reports; it launches nothing.  Returns FQ_OK, or the status fq_gemm would return for an
 * invalid shape.
 */
int fq_gemm_describe(int64_t M, int64_t N, int64_t K, int bits, int group_size, char* buf,
                     size_t buf_bytes);

/*
 * fq_stream_read_probe -- measurement helper, not part of the method: one kernel that reads
 * `bytes` bytes of device memory (16 bytes per lane, grid-stride, 256 blocks of 768 threads: the
 * launch shape of the small-M product) and writes one 32-bit checksum word per block to `sink`
 * (device, >= 1024 bytes).  Timed by the caller, it gives the
 * rate at which this GPU streams a buffer through a kernel that does nothing else: the ceiling the
 * small-M product is compared with next to the vendor's peak.  `bytes` must be a multiple of 16.
 * Errors: FQ_ERR_INVALID_ARG, FQ_ERR_HIP.
 */
int fq_stream_read_probe(const void* buf, size_t bytes, void* sink, void* stream);

/*
 * fq_mfma_rate_probe -- measurement helper, not part of the method: one kernel (1024 blocks of 8 waves) that
 * runs the MFMA loop of the 128-row shape of the large-M product (per wave and iteration 96
 * v_mfma_f32_16x16x32_f16: 4 k-steps x 8 row tiles x 3 column tiles) on the caller's operand VALUES and nothing
 * else: no global loads in the loop, no conversions, no barrier; with lds_reads != 0 one 16-byte fragment
 * read from LDS per lane and three MFMAs, as in the product.  The clock this GPU holds under load follows the
 * switching activity of the operands, so the rate of this loop on operands distributed like the product's
 * (and not the vendor's peak, which it reaches on all-zero operands only) is what the matrix pipes can
 * deliver to the product; the caller times it.  With int8 != 0 the loop uses the integer path's instruction
 * (v_mfma_i32_16x16x64_i8) on the same bytes read as int8 values.
 *   operands   in   device, >= fq_mfma_rate_probe_operand_bytes() bytes of binary16 (or int8) values, read as
 *                   they are
 *   sink       out  device, >= fq_mfma_rate_probe_sink_bytes() bytes (one binary32 checksum per thread)
 * One launch performs fq_mfma_rate_probe_flops(iterations, int8) operations (2 per multiply-add).
 * Errors: FQ_ERR_INVALID_ARG (NULL pointer, iterations outside 1 .. 2^16: a launch stays below a second), FQ_ERR_WORKSPACE (a buffer is too
 * small), FQ_ERR_HIP.
 */
size_t fq_mfma_rate_probe_operand_bytes(void);
size_t fq_mfma_rate_probe_sink_bytes(void);
double fq_mfma_rate_probe_flops(int iterations, int int8);
int fq_mfma_rate_probe(const void* operands, size_t operand_bytes, void* sink, size_t sink_bytes, int iterations,
                       int lds_reads, int int8, void* stream);

/* Human-readable name of a status code (static string, never NULL). */
const char* fq_status_string(int status);

/* Library version, "major.minor". */
const char* fq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FQ_H_ */
