// Host side of the product: the plan (which kernel, which block shape) and the entry points
// that dispatch on activation type and code width.  The kernels themselves are instantiated
// in fq_gemm_<type>_<bits>.hip.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fq_gemm_config.h"
#include "fq_internal.h"
#include "fq_layout.h"


using namespace fqd;

#define FQ_DECLARE_GEMM(ACT, BITS)                                                                         \
    int fq_launch_typed_##ACT##_##BITS(const void* A, int64_t M, int64_t N, int64_t K, const void* codes,  \
                                       const void* scales, int g, void* C, void* workspace,                \
                                       const fq_gemm_plan& plan, hipStream_t stream);                      \
    int fq_launch_grouped_typed_##ACT##_##BITS(const void* A, const int32_t* offsets, int E, int64_t N,    \
                                               int64_t K, const void* codes, const void* scales, int g,    \
                                               void* C, hipStream_t stream);
FQ_DECLARE_GEMM(0, 4)
FQ_DECLARE_GEMM(0, 8)
FQ_DECLARE_GEMM(1, 4)
FQ_DECLARE_GEMM(1, 8)

fq_gemm_plan fq_plan_gemm(int64_t M, int64_t N, int64_t K, int bits, int g) {
    (void)g;
    fq_gemm_plan p = {};
    const int kblk = fq_kblk(bits);
    const int KB = (int)(K / kblk);
    const int ntiles = (int)(N / FQ_NTILE);
    if (M <= 16) {
        // One block per compute unit, all resident at once.  Candidates are scored by how evenly
        // the column tiles fill 256 blocks, by the bytes a compute unit keeps in flight
        // (waves x NT KiB x ring depth, ~64 KiB saturates), and by how many activation units a
        // lane must stage (fewer registers); ties keep the earlier variant.
        p.kind = 0;
        p.mt = 1;
        const int kc = kblk / 8;
        const double f_nt[4] = {0.0, 0.93, 0.97, 1.0};
        double best = -1.0;
        for (int v = 0; v < 4; ++v) {
            const SkinnyVariant sv = SKINNY_VARIANTS[v];
            for (int gp = 1; gp <= sv.maxw; ++gp) {
                const int tb = sv.nt * gp;
                const int64_t blocks = (ntiles + tb - 1) / tb;
                const int64_t rounds = (blocks + 255) / 256;
                const double eff = (double)ntiles / (double)(rounds * 256 * tb);
                const int need = (int)M * kc;
                const int au = need <= 64 * gp ? 1 : (need <= 128 * gp ? 2 : (need <= 256 * gp ? 4 : 0));
                if (au == 0) continue;
                int kw = sv.maxw / gp;
                if (kw > 8) kw = 8;
                if (kw > KB) kw = KB;
                if (kw < 1) continue;
                const int waves = gp * kw;
                const double inflight = (double)waves * sv.nt * sv.depth;   // KiB
                double score = eff * eff * (inflight >= 64.0 ? 1.0 : sqrt(inflight / 64.0)) * f_nt[sv.nt];
                score /= 1.0 + 0.1 * (double)(rounds - 1);   // a single resident round beats several
                score *= au == 1 ? 1.0 : (au == 2 ? 0.8 : 0.6);
                if (waves < 6) score *= 0.85;
                if (score > best + 1e-9) {
                    best = score;
                    p.variant = v;
                    p.gp = gp;
                    p.kw = kw;
                    p.au = au;
                    p.waves = waves;
                }
            }
        }
        const SkinnyVariant sv = SKINNY_VARIANTS[p.variant];
        const int64_t blocks = (ntiles + sv.nt * p.gp - 1) / (sv.nt * p.gp);
        const int SB = (KB + p.kw - 1) / p.kw;
        int gs = 1;
        if (blocks <= 128) gs = (int)(256 / blocks);
        if (gs > 8) gs = 8;
        if (gs > SB) gs = SB;
        p.splits = gs;
        p.kb_per_split = 0;
    } else {
        // Tiled MFMA kernel: BM = 16 * mt rows per block, 64 columns per wave.
        p.kind = 1;
        p.mt = M <= 32 ? 2 : (M <= 64 ? 4 : 8);
        const int bm = p.mt * 16;
        const int64_t nbm = (M + bm - 1) / bm;
        const int64_t blocks8 = ((ntiles + 8 * MMA_NT - 1) / (8 * MMA_NT)) * nbm;
        const int64_t blocks4 = ((ntiles + 4 * MMA_NT - 1) / (4 * MMA_NT)) * nbm;
        p.waves = blocks8 >= 512 ? 8 : 4;
        const int64_t blocks = p.waves == 8 ? blocks8 : blocks4;
        int splits = 1;
        if (blocks < 256) splits = (int)((512 + blocks - 1) / blocks);
        if (splits > 8) splits = 8;
        if (splits > KB) splits = KB;
        const int kbs = (KB + splits - 1) / splits;
        p.kb_per_split = kbs;
        p.splits = (KB + kbs - 1) / kbs;
    }
    return p;
}

int fq_launch_gemm(const void* A, int act, int64_t M, int64_t N, int64_t K, const void* codes,
                   const void* scales, int bits, int g, void* C, void* workspace, hipStream_t stream) {
    const fq_gemm_plan plan = fq_plan_gemm(M, N, K, bits, g);
    if (act == FQ_F16) {
        if (bits == 4) return fq_launch_typed_0_4(A, M, N, K, codes, scales, g, C, workspace, plan, stream);
        return fq_launch_typed_0_8(A, M, N, K, codes, scales, g, C, workspace, plan, stream);
    }
    if (bits == 4) return fq_launch_typed_1_4(A, M, N, K, codes, scales, g, C, workspace, plan, stream);
    return fq_launch_typed_1_8(A, M, N, K, codes, scales, g, C, workspace, plan, stream);
}

int fq_launch_gemm_grouped(const void* A, int act, const int32_t* offsets, int E, int64_t N, int64_t K,
                           const void* codes, const void* scales, int bits, int g, void* C,
                           hipStream_t stream) {
    if (act == FQ_F16) {
        if (bits == 4) return fq_launch_grouped_typed_0_4(A, offsets, E, N, K, codes, scales, g, C, stream);
        return fq_launch_grouped_typed_0_8(A, offsets, E, N, K, codes, scales, g, C, stream);
    }
    if (bits == 4) return fq_launch_grouped_typed_1_4(A, offsets, E, N, K, codes, scales, g, C, stream);
    return fq_launch_grouped_typed_1_8(A, offsets, E, N, K, codes, scales, g, C, stream);
}
