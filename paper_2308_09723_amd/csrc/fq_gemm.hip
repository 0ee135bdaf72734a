// Fused dequantise-and-multiply kernels for gfx950 (section 4.1, "GPU kernel
// implementations": int4/int8 weights with a matrix of scales, fp16/bf16 activations,
// floating-point matrix-core math, output in the activation type).
//
// Orientation: every product is computed as 16x16 tiles of C^T with
// v_mfma_f32_16x16x32_{f16,bf16}.  The WEIGHTS are the first MFMA operand (its 16 rows are
// 16 output columns n), the ACTIVATIONS the second (its 16 columns are 16 rows m of A).
// A lane's 16-byte record of the packed layout is, after the integer->float step, directly
// its slice of the first operand: weights never pass through LDS.  The result tile leaves
// lane l with C[m = l % 16][n = 4 (l / 16) + 0..3], i.e. four consecutive columns of one row.
//
// Numerics: the integer codes are converted EXACTLY to the activation type (bf16 carries
// them with a constant offset that is removed in binary32), multiplied on the matrix cores
// with binary32 accumulation over one scale group (or one k-block), and the group's scale
// is applied to that partial sum in binary32.  Nothing is rounded to 16 bits before the
// final store.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fq_gemm_kernels.h"

namespace {

using namespace fqk;

// ------------------------------------------------------------------------------ dispatch
constexpr int TILE_NT = 4;

// Small-M kernel variants that are compiled in: (NT column tiles per wave, ring DEPTH,
// register class = maximum waves per block).  The plan picks one of them plus the run-time
// block shape (GP column groups x KW k-workers).
//   variant 0: NT 3, DEPTH 2, up to 12 waves     variant 1: NT 3, DEPTH 3, up to 8 waves
//   variant 2: NT 1, DEPTH 4, up to 12 waves     variant 3: NT 2, DEPTH 3, up to 12 waves
struct SkinnyVariant { int nt, depth, maxw; };
constexpr SkinnyVariant SKINNY_VARIANTS[4] = {{3, 2, 12}, {3, 3, 8}, {1, 4, 12}, {2, 3, 12}};

template <int ACT, int BITS, int NT, int DEPTH, int MAXW, int AU>
int launch_skinny(const void* A, int64_t M, int64_t N, int64_t K, const void* codes, const void* scales, int g,
                  void* C, float* partial, const fq_gemm_plan& plan, hipStream_t stream) {
    const int kblk = fq_kblk(BITS);
    const bool per_step = (g % kblk) != 0;
    const int ntiles = (int)(N / FQ_NTILE);
    const int ngroups = (ntiles + NT - 1) / NT;
    const int bgroups = (ngroups + plan.gp - 1) / plan.gp;
    const int kc = kblk / 8;
    const size_t lds_act = (size_t)2 * plan.kw * kc * FQ_SK_PITCH * 16;
    const size_t lds_red = (size_t)plan.gp * plan.kw * NT * 64 * 16;
    const size_t lds = lds_act > lds_red ? lds_act : lds_red;
    const uint32_t g32 = (uint32_t)(g / 32);
    const uint32_t g32_recip = (uint32_t)((((uint64_t)1 << 32) + g32 - 1) / g32);   // unused when g32 == 1
    auto kern = per_step ? fq_gemm_skinny_kernel<ACT, BITS, NT, DEPTH, true, MAXW, AU>
                         : fq_gemm_skinny_kernel<ACT, BITS, NT, DEPTH, false, MAXW, AU>;
    if (lds > 65536) {
        // more than the default dynamic LDS limit: raise it for this kernel (up to the 160 KiB of a CU)
        if (lds > 160 * 1024) return FQ_ERR_UNSUPPORTED;
        static bool raised[2] = {false, false};   // per instantiation: [per_step]
        if (!raised[per_step ? 1 : 0]) {
            if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024) != hipSuccess)
                return FQ_ERR_HIP;
            raised[per_step ? 1 : 0] = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(bgroups * plan.splits)), dim3((unsigned)(plan.gp * plan.kw * 64)),
                       lds, stream, (const uint16_t*)A, (const u32x4*)codes, (const uint16_t*)scales,
                       (uint16_t*)C, partial, (int)M, (int)N, (int)K, g32, g32_recip, plan.gp, plan.kw,
                       plan.splits);
    return FQ_OK;
}

template <int ACT, int BITS, int NT, int DEPTH, int MAXW>
int launch_skinny_au(const void* A, int64_t M, int64_t N, int64_t K, const void* codes, const void* scales,
                     int g, void* C, float* partial, const fq_gemm_plan& plan, hipStream_t stream) {
    switch (plan.au) {
        case 1: return launch_skinny<ACT, BITS, NT, DEPTH, MAXW, 1>(A, M, N, K, codes, scales, g, C, partial, plan, stream);
        case 2: return launch_skinny<ACT, BITS, NT, DEPTH, MAXW, 2>(A, M, N, K, codes, scales, g, C, partial, plan, stream);
        default: return launch_skinny<ACT, BITS, NT, DEPTH, MAXW, 4>(A, M, N, K, codes, scales, g, C, partial, plan, stream);
    }
}

template <int ACT, int BITS>
int launch_typed(const void* A, int64_t M, int64_t N, int64_t K, const void* codes, const void* scales,
                 int g, void* C, void* workspace, const fq_gemm_plan& plan, hipStream_t stream) {
    const int kblk = fq_kblk(BITS);
    const bool per_step = (g % kblk) != 0;
    const int ntiles = (int)(N / FQ_NTILE);
    float* partial = (float*)workspace;
    if (plan.kind == 0) {
        int st;
        switch (plan.variant) {
            case 0: st = launch_skinny_au<ACT, BITS, 3, 2, 12>(A, M, N, K, codes, scales, g, C, partial, plan, stream); break;
            case 1: st = launch_skinny_au<ACT, BITS, 3, 3, 8>(A, M, N, K, codes, scales, g, C, partial, plan, stream); break;
            case 2: st = launch_skinny_au<ACT, BITS, 1, 4, 12>(A, M, N, K, codes, scales, g, C, partial, plan, stream); break;
            default: st = launch_skinny_au<ACT, BITS, 2, 3, 12>(A, M, N, K, codes, scales, g, C, partial, plan, stream); break;
        }
        if (st != FQ_OK) return st;
    } else {
        const int bm = plan.mt * 16;
        dim3 grid((unsigned)((ntiles + 4 * TILE_NT - 1) / (4 * TILE_NT)), (unsigned)((M + bm - 1) / bm),
                  (unsigned)plan.splits);
        fq_group_items none;
        none.count = 0;
#define FQ_TILE_LAUNCH(MT_)                                                                           \
    do {                                                                                              \
        auto kern = per_step ? fq_gemm_tile_kernel<ACT, BITS, MT_, TILE_NT, true, false>              \
                             : fq_gemm_tile_kernel<ACT, BITS, MT_, TILE_NT, false, false>;            \
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, (const uint16_t*)A, (const u32x4*)codes, \
                           (const uint16_t*)scales, (uint16_t*)C, partial, (int)M, (int)N, (int)K, g, \
                           plan.kb_per_split, plan.splits, (int64_t)0, (int64_t)0, none);             \
    } while (0)
        if (plan.mt == 1) FQ_TILE_LAUNCH(1);
        else if (plan.mt == 2) FQ_TILE_LAUNCH(2);
        else FQ_TILE_LAUNCH(4);
#undef FQ_TILE_LAUNCH
    }
    if (plan.splits > 1) {
        const int64_t MN = M * N;
        dim3 grid((unsigned)((MN / 4 + 255) / 256));
        hipLaunchKernelGGL(fq_reduce_kernel<ACT>, grid, dim3(256), 0, stream, (const float*)partial,
                           plan.splits, MN, (uint16_t*)C);
    }
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}

template <int ACT, int BITS>
int launch_grouped_typed(const void* A, const int32_t* offsets, int E, int64_t N, int64_t K,
                         const void* codes, const void* scales, int g, void* C, hipStream_t stream) {
    constexpr int MT = 4;
    constexpr int BM = MT * 16;
    const int kblk = fq_kblk(BITS);
    const bool per_step = (g % kblk) != 0;
    const int ntiles = (int)(N / FQ_NTILE);
    const int KB = (int)(K / kblk);
    const int64_t codes_stride16 = (int64_t)(K * N * BITS / 8) / 16;
    const int64_t scales_stride = (K / g) * N;
    fq_group_items items;
    items.count = 0;
    auto flush_items = [&]() -> int {
        if (items.count == 0) return FQ_OK;
        dim3 grid((unsigned)((ntiles + 4 * TILE_NT - 1) / (4 * TILE_NT)), (unsigned)items.count, 1u);
        auto kern = per_step ? fq_gemm_tile_kernel<ACT, BITS, MT, TILE_NT, true, true>
                             : fq_gemm_tile_kernel<ACT, BITS, MT, TILE_NT, false, true>;
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, (const uint16_t*)A, (const u32x4*)codes,
                           (const uint16_t*)scales, (uint16_t*)C, (float*)nullptr, 0, (int)N, (int)K, g, KB, 1,
                           codes_stride16, scales_stride, items);
        items.count = 0;
        return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
    };
    for (int e = 0; e < E; ++e) {
        for (int32_t r = offsets[e]; r < offsets[e + 1]; r += BM) {
            const int i = items.count++;
            items.row0[i] = r;
            items.rows[i] = (int16_t)min(BM, offsets[e + 1] - r);
            items.expert[i] = (int16_t)e;
            if (items.count == 256) {
                const int st = flush_items();
                if (st != FQ_OK) return st;
            }
        }
    }
    return flush_items();
}

}  // namespace

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
        p.kind = 1;
        p.waves = 4;
        p.mt = M <= 32 ? 2 : 4;
        const int bm = p.mt * 16;
        const int64_t blocks = ((ntiles + 4 * TILE_NT - 1) / (4 * TILE_NT)) * ((M + bm - 1) / bm);
        int splits = 1;
        if (blocks < 512) splits = (int)((512 + blocks - 1) / blocks);
        if (splits > 8) splits = 8;
        if (splits > KB) splits = KB;
        int kbs = (KB + splits - 1) / splits;
        p.kb_per_split = kbs;
        p.splits = (KB + kbs - 1) / kbs;
    }
    return p;
}

int fq_launch_gemm(const void* A, int act, int64_t M, int64_t N, int64_t K, const void* codes,
                   const void* scales, int bits, int g, void* C, void* workspace, hipStream_t stream) {
    const fq_gemm_plan plan = fq_plan_gemm(M, N, K, bits, g);
    if (act == FQ_F16) {
        if (bits == 4) return launch_typed<FQ_F16, 4>(A, M, N, K, codes, scales, g, C, workspace, plan, stream);
        return launch_typed<FQ_F16, 8>(A, M, N, K, codes, scales, g, C, workspace, plan, stream);
    }
    if (bits == 4) return launch_typed<FQ_BF16, 4>(A, M, N, K, codes, scales, g, C, workspace, plan, stream);
    return launch_typed<FQ_BF16, 8>(A, M, N, K, codes, scales, g, C, workspace, plan, stream);
}

int fq_launch_gemm_grouped(const void* A, int act, const int32_t* offsets, int E, int64_t N, int64_t K,
                           const void* codes, const void* scales, int bits, int g, void* C,
                           hipStream_t stream) {
    if (act == FQ_F16) {
        if (bits == 4) return launch_grouped_typed<FQ_F16, 4>(A, offsets, E, N, K, codes, scales, g, C, stream);
        return launch_grouped_typed<FQ_F16, 8>(A, offsets, E, N, K, codes, scales, g, C, stream);
    }
    if (bits == 4) return launch_grouped_typed<FQ_BF16, 4>(A, offsets, E, N, K, codes, scales, g, C, stream);
    return launch_grouped_typed<FQ_BF16, 8>(A, offsets, E, N, K, codes, scales, g, C, stream);
}
