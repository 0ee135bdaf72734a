// C ABI of libfq: argument validation on the host, then dispatch to the launchers.
// Every check happens before the first HIP call, so invalid calls never touch the GPU.
#include <hip/hip_runtime.h>
#include <mutex>
#include <stdint.h>
#include <stdio.h>

#include "fq_internal.h"
#include "fq_layout.h"

namespace {

bool bits_ok(int bits) { return bits == 3 || bits == 4 || bits == 8; }

// Returns FQ_OK and the effective group size in *g_eff, or an error status.
int check_shape(int64_t K, int64_t N, int bits, int group_size, int* g_eff) {
    if (!bits_ok(bits) || K <= 0 || N <= 0 || group_size < 0) return FQ_ERR_INVALID_ARG;
    const int64_t g = (group_size == 0) ? K : (int64_t)group_size;
    if (g > K || K % g != 0) return FQ_ERR_INVALID_ARG;
    if (K > (int64_t)1 << 24 || N > (int64_t)1 << 24) return FQ_ERR_UNSUPPORTED;
    if (N % FQ_NTILE != 0 || K % fq_kblk(bits) != 0) return FQ_ERR_UNSUPPORTED;
    if (g % 32 != 0) return FQ_ERR_UNSUPPORTED;
    if (K / g > 65535) return FQ_ERR_UNSUPPORTED;
    if (g_eff) *g_eff = (int)g;
    return FQ_OK;
}

int halving_levels(int64_t g_top, int g_min) {
    int levels = 0;
    int64_t g = g_top;
    while (g % 2 == 0 && g / 2 >= g_min) {
        g /= 2;
        ++levels;
    }
    return levels;
}

}  // namespace

extern "C" {

size_t fq_codes_bytes(int64_t K, int64_t N, int bits) {
    if (!bits_ok(bits) || K <= 0 || N <= 0) return 0;
    return (size_t)(K * N * bits / 8);
}

size_t fq_scales_bytes(int64_t K, int64_t N, int group_size) {
    if (K <= 0 || N <= 0 || group_size < 0) return 0;
    const int64_t g = group_size == 0 ? K : group_size;
    if (g > K || K % g != 0) return 0;
    return (size_t)((K / g) * N * 2);
}

size_t fq_gemm_workspace_bytes_for(int64_t M, int64_t N, int64_t K, int bits, int group_size, int act_dtype,
                                   int scale_format) {
    int g = 0;
    if (M <= 0 || check_shape(K, N, bits, group_size, &g) != FQ_OK) return 0;
    const fq_gemm_plan plan = fq_plan_gemm(M, N, K, bits, g);
    size_t need = fq_partial_bytes(plan, M, N);
    if (fq_via_f16(act_dtype, scale_format, plan, N)) need += fq_a16_bytes(M, K) + fq_rowscale_bytes(M);
    return need;
}

size_t fq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int bits, int group_size) {
    // the largest need over the activation types and scale formats
    return fq_gemm_workspace_bytes_for(M, N, K, bits, group_size, FQ_BF16, FQ_SCALE_F16);
}

size_t fq_gemm_grouped_workspace_bytes(int64_t total_rows, int E, int64_t N, int64_t K, int bits,
                                       int group_size) {
    (void)total_rows; (void)E; (void)N; (void)K; (void)bits; (void)group_size;
    return 0;
}

int fq_quantize_sf(const void* W_f16, int64_t K, int64_t N, int bits, int group_size, int scale_format,
                   void* codes, void* scales, void* stream) {
    if (!W_f16 || !codes || !scales) return FQ_ERR_INVALID_ARG;
    if (scale_format != FQ_SCALE_F16 && scale_format != FQ_SCALE_BF16) return FQ_ERR_INVALID_ARG;
    int g = 0;
    const int st = check_shape(K, N, bits, group_size, &g);
    if (st != FQ_OK) return st;
    return fq_launch_quantize(W_f16, K, N, bits, g, scale_format, codes, scales, (hipStream_t)stream);
}

int fq_quantize(const void* W_f16, int64_t K, int64_t N, int bits, int group_size, void* codes,
                void* scales_f16, void* stream) {
    return fq_quantize_sf(W_f16, K, N, bits, group_size, FQ_SCALE_F16, codes, scales_f16, stream);
}

int fq_unpack(const void* codes, int64_t K, int64_t N, int bits, int8_t* q, void* stream) {
    if (!codes || !q) return FQ_ERR_INVALID_ARG;
    const int st = check_shape(K, N, bits, 0, nullptr);
    if (st != FQ_OK) return st;
    return fq_launch_unpack(codes, K, N, bits, q, (hipStream_t)stream);
}

size_t fq_choose_group_workspace_bytes(int64_t K, int64_t N, int g_start, int g_min) {
    if (K <= 0 || N <= 0 || g_start < 0 || g_min <= 0) return 0;
    const int64_t g_top = g_start == 0 ? K : g_start;
    if (g_top > K || K % g_top != 0) return 0;
    const int levels = halving_levels(g_top, g_min);
    const int64_t f = g_top >> levels;
    return (size_t)(256 + (K / f) * N * 2);
}

int fq_choose_group(const void* W_f16, int64_t K, int64_t N, int g_start, int g_min, float alpha,
                    int* g_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!W_f16 || !g_out || K <= 0 || N <= 0 || g_start < 0 || g_min <= 0) return FQ_ERR_INVALID_ARG;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return FQ_ERR_INVALID_ARG;
    const int64_t g_top = g_start == 0 ? K : g_start;
    if (g_top > K || K % g_top != 0) return FQ_ERR_INVALID_ARG;
    // (the abs-max kernel reads eight columns per lane)
    if (N % FQ_NTILE != 0 || K > (int64_t)1 << 24 || N > (int64_t)1 << 24) return FQ_ERR_UNSUPPORTED;
    const int levels = halving_levels(g_top, g_min);
    if (levels == 0) {
        *g_out = (int)g_top;
        return FQ_OK;
    }
    const int64_t f = g_top >> levels;
    if (levels > 24 || K / f > 65535 || K / g_top > 65535) return FQ_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < fq_choose_group_workspace_bytes(K, N, g_start, g_min))
        return FQ_ERR_WORKSPACE;
    int flags[64];
    const int st = fq_launch_choose_group(W_f16, K, N, (int)g_top, levels, alpha, flags, workspace,
                                          (hipStream_t)stream);
    if (st != FQ_OK) return st;
    int64_t g = g_top;
    for (int d = 0; d < levels; ++d) {
        if (!flags[d]) break;
        g /= 2;
    }
    *g_out = (int)g;
    return FQ_OK;
}

size_t fq_quant_error_workspace_bytes(int64_t K, int64_t N) {
    if (K <= 0 || N <= 0) return 0;
    return (size_t)(16 + 16 * fq_quant_error_blocks(K, N));
}

int fq_quant_error(const void* W_f16, int64_t K, int64_t N, int bits, int group_size, const void* codes,
                   const void* scales_f16, double* sse_out, double* max_abs_out, void* workspace,
                   size_t workspace_bytes, void* stream) {
    return fq_quant_error_sf(W_f16, K, N, bits, group_size, FQ_SCALE_F16, codes, scales_f16, sse_out, max_abs_out,
                             workspace, workspace_bytes, stream);
}

int fq_quant_error_sf(const void* W_f16, int64_t K, int64_t N, int bits, int group_size, int scale_format,
                      const void* codes, const void* scales_f16, double* sse_out, double* max_abs_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
    if (!W_f16 || !codes || !scales_f16 || !sse_out || !max_abs_out) return FQ_ERR_INVALID_ARG;
    if (scale_format != FQ_SCALE_F16 && scale_format != FQ_SCALE_BF16) return FQ_ERR_INVALID_ARG;
    int g = 0;
    const int st = check_shape(K, N, bits, group_size, &g);
    if (st != FQ_OK) return st;
    if (!workspace || workspace_bytes < fq_quant_error_workspace_bytes(K, N)) return FQ_ERR_WORKSPACE;
    double out[2] = {0.0, 0.0};
    const int rc = fq_launch_quant_error(W_f16, K, N, bits, g, scale_format, codes, scales_f16, out, workspace,
                                         (hipStream_t)stream);
    if (rc != FQ_OK) return rc;
    *sse_out = out[0];
    *max_abs_out = out[1];
    return FQ_OK;
}

// internal activation kind: FQ_F16, FQ_BF16, or 2 = bf16 activations with bf16 scales; -1 = refuse
static int act_kind(int act_dtype, int scale_format, int* status) {
    *status = FQ_OK;
    if (act_dtype != FQ_F16 && act_dtype != FQ_BF16) *status = FQ_ERR_INVALID_ARG;
    else if (scale_format != FQ_SCALE_F16 && scale_format != FQ_SCALE_BF16) *status = FQ_ERR_INVALID_ARG;
    else if (scale_format == FQ_SCALE_BF16 && act_dtype != FQ_BF16) *status = FQ_ERR_UNSUPPORTED;
    if (*status != FQ_OK) return -1;
    return scale_format == FQ_SCALE_BF16 ? 2 : act_dtype;
}

int fq_gemm(const void* A, int act_dtype, int64_t M, int64_t N, int64_t K, const void* codes,
            const void* scales_f16, int bits, int group_size, void* C, void* workspace,
            size_t workspace_bytes, void* stream) {
    return fq_gemm_sf(A, act_dtype, M, N, K, codes, scales_f16, FQ_SCALE_F16, bits, group_size, C, workspace,
                      workspace_bytes, stream);
}

int fq_gemm_sf(const void* A, int act_dtype, int64_t M, int64_t N, int64_t K, const void* codes,
               const void* scales_f16, int scale_format, int bits, int group_size, void* C, void* workspace,
               size_t workspace_bytes, void* stream) {
    if (M < 0) return FQ_ERR_INVALID_ARG;
    int kst = FQ_OK;
    const int kind = act_kind(act_dtype, scale_format, &kst);
    if (kst == FQ_ERR_INVALID_ARG) return kst;
    int g = 0;
    const int st = check_shape(K, N, bits, group_size, &g);
    if (st != FQ_OK) return st;
    if (kst != FQ_OK) return kst;
    if (M == 0) return FQ_OK;
    if (!A || !codes || !scales_f16 || !C) return FQ_ERR_INVALID_ARG;
    if (M > (int64_t)1 << 24) return FQ_ERR_UNSUPPORTED;
    const size_t need = fq_gemm_workspace_bytes_for(M, N, K, bits, group_size, act_dtype, scale_format);
    if (need > 0 && (!workspace || workspace_bytes < need)) return FQ_ERR_WORKSPACE;
    return fq_launch_gemm(A, kind, M, N, K, codes, scales_f16, bits, g, C, workspace,
                          (hipStream_t)stream);
}

}  // extern "C"

// Scratch of fq_gemm_noalloc: a file-scope device array (every GPU the library runs on holds its own copy,
// at its own address, until the process ends).  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address kernels may use is asked for once per device and kept here.
static __device__ __align__(256) unsigned char scratch[FQ_NOALLOC_SCRATCH_BYTES];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[64];

// Device address of `scratch` on the current device, or nullptr (with *status set) on failure.
void* scratch_of_current_device(int* status) {
    int dev = 0;
    *status = FQ_OK;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        *status = FQ_ERR_HIP;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            *status = FQ_ERR_HIP;
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

int fq_gemm_noalloc(const void* A, int act_dtype, int64_t M, int64_t N, int64_t K, const void* codes,
                    const void* scales_f16, int bits, int group_size, void* C, void* stream) {
    if (M < 0) return FQ_ERR_INVALID_ARG;
    int kst = FQ_OK;
    const int kind = act_kind(act_dtype, FQ_SCALE_F16, &kst);
    if (kst != FQ_OK) return kst;
    int g = 0;
    const int st = check_shape(K, N, bits, group_size, &g);
    if (st != FQ_OK) return st;
    if (M == 0) return FQ_OK;
    if (!A || !codes || !scales_f16 || !C) return FQ_ERR_INVALID_ARG;
    if (M > (int64_t)1 << 24) return FQ_ERR_UNSUPPORTED;
    const size_t need = fq_gemm_workspace_bytes_for(M, N, K, bits, group_size, act_dtype, FQ_SCALE_F16);
    if (need > (size_t)FQ_NOALLOC_SCRATCH_BYTES) return FQ_ERR_WORKSPACE;   // beyond the static scratch
    void* ws = nullptr;
    if (need > 0) {
        int sst = FQ_OK;
        ws = scratch_of_current_device(&sst);
        if (!ws) return sst;
    }
    // Nothing in the scratch has to start at zero: every partial sum and every rewritten activation row a
    // kernel of this call reads was written by an earlier kernel of the same call.
    return fq_launch_gemm(A, kind, M, N, K, codes, scales_f16, bits, g, C, ws, (hipStream_t)stream);
}

size_t fq_gemm_noalloc_scratch_bytes(void) { return (size_t)FQ_NOALLOC_SCRATCH_BYTES; }

int fq_gemm_grouped(const void* A, int act_dtype, const int32_t* offsets_host, int E, int64_t N,
                    int64_t K, const void* codes, const void* scales_f16, int bits, int group_size,
                    void* C, void* workspace, size_t workspace_bytes, void* stream) {
    return fq_gemm_grouped_sf(A, act_dtype, offsets_host, E, N, K, codes, scales_f16, FQ_SCALE_F16, bits,
                              group_size, C, workspace, workspace_bytes, stream);
}

int fq_gemm_grouped_sf(const void* A, int act_dtype, const int32_t* offsets_host, int E, int64_t N,
                       int64_t K, const void* codes, const void* scales_f16, int scale_format, int bits,
                       int group_size, void* C, void* workspace, size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    if (!offsets_host || E < 0) return FQ_ERR_INVALID_ARG;
    int kst = FQ_OK;
    const int kind = act_kind(act_dtype, scale_format, &kst);
    if (kst != FQ_OK) return kst;
    if (E > 256) return FQ_ERR_UNSUPPORTED;
    int g = 0;
    const int st = check_shape(K, N, bits, group_size, &g);
    if (st != FQ_OK) return st;
    if (E == 0) return FQ_OK;
    if (offsets_host[0] != 0) return FQ_ERR_INVALID_ARG;
    for (int e = 0; e < E; ++e)
        if (offsets_host[e + 1] < offsets_host[e]) return FQ_ERR_INVALID_ARG;
    if (offsets_host[E] == 0) return FQ_OK;
    if (!A || !codes || !scales_f16 || !C) return FQ_ERR_INVALID_ARG;
    return fq_launch_gemm_grouped(A, kind, offsets_host, E, N, K, codes, scales_f16, bits, g, C,
                                  (hipStream_t)stream);
}

int fq_gemm_describe(int64_t M, int64_t N, int64_t K, int bits, int group_size, char* buf,
                     size_t buf_bytes) {
    if (!buf || buf_bytes == 0 || M < 0) return FQ_ERR_INVALID_ARG;
    int g = 0;
    const int st = check_shape(K, N, bits, group_size, &g);
    if (st != FQ_OK) return st;
    if (M == 0) {
        snprintf(buf, buf_bytes, "empty");
        return FQ_OK;
    }
    const fq_gemm_plan p = fq_plan_gemm(M, N, K, bits, g);
    if (p.kind == 0)
        snprintf(buf, buf_bytes, "small-m variant=%d gp=%d kw=%d au=%d waves=%d splits=%d", p.variant, p.gp,
                 p.kw, p.au, p.waves, p.splits);
    else
        snprintf(buf, buf_bytes, "tiled mt=%d waves=%d splits=%d kb_per_split=%d tail=%dx%d", p.mt, p.waves, p.splits,
                 p.kb_per_split, p.tail_tiles, p.tail_tiles > 0 ? p.tail_splits : 1);
    return FQ_OK;
}

int fq_stream_read_probe(const void* buf, size_t bytes, void* sink, void* stream) {
    if (!buf || !sink || bytes == 0 || bytes % 16 != 0) return FQ_ERR_INVALID_ARG;
    return fq_launch_stream_read_probe(buf, bytes, sink, (hipStream_t)stream);
}

size_t fq_mfma_rate_probe_operand_bytes(void) { return fq_mfma_probe_operand_bytes(); }
size_t fq_mfma_rate_probe_sink_bytes(void) { return fq_mfma_probe_sink_bytes(); }
double fq_mfma_rate_probe_flops(int iterations, int int8) {
    return iterations > 0 ? fq_mfma_probe_flops(iterations, int8 != 0) : 0.0;
}

int fq_mfma_rate_probe(const void* operands, size_t operand_bytes, void* sink, size_t sink_bytes, int iterations,
                       int lds_reads, int int8, void* stream) {
    if (!operands || !sink || iterations <= 0 || iterations > (1 << 16)) return FQ_ERR_INVALID_ARG;
    if (operand_bytes < fq_mfma_probe_operand_bytes() || sink_bytes < fq_mfma_probe_sink_bytes()) return FQ_ERR_WORKSPACE;
    return fq_launch_mfma_rate_probe(operands, sink, iterations, lds_reads != 0, int8 != 0, (hipStream_t)stream);
}

const char* fq_status_string(int status) {
    switch (status) {
        case FQ_OK: return "FQ_OK";
        case FQ_ERR_INVALID_ARG: return "FQ_ERR_INVALID_ARG";
        case FQ_ERR_UNSUPPORTED: return "FQ_ERR_UNSUPPORTED";
        case FQ_ERR_WORKSPACE: return "FQ_ERR_WORKSPACE";
        case FQ_ERR_HIP: return "FQ_ERR_HIP";
        default: return "FQ_ERR_UNKNOWN";
    }
}

const char* fq_version(void) { return "0.1"; }

}  // extern "C"
