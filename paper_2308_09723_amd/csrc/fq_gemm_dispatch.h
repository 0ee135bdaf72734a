// Host-side dispatch templates of the product kernels (included by the per-type translation
// units fq_gemm_f16_4.hip ... so that they compile in parallel).
#ifndef FQ_GEMM_DISPATCH_H_
#define FQ_GEMM_DISPATCH_H_

#include <math.h>
#include <stdint.h>
#include <atomic>

#include "fq_gemm_config.h"
#include "fq_gemm_kernels.h"

namespace fqd {

using namespace fqk;

// Kernels that need more than the default 64 KiB of dynamic LDS have their limit raised to the
// 160 KiB of a compute unit, once per (kernel instantiation, device): `done` holds one bit per device.
inline int raise_lds_limit(const void* kern, std::atomic<uint64_t>& done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return FQ_ERR_HIP;
    const uint64_t bit = (uint64_t)1 << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return FQ_OK;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
        return FQ_ERR_HIP;
    done.fetch_or(bit, std::memory_order_release);
    return FQ_OK;
}

template <int ACT, int BITS, int NT, int DEPTH, int MAXW, int AU>
int launch_skinny(const void* A, int64_t M, int64_t N, int64_t K, const void* codes, const void* scales, int g,
                  void* C, float* partial, const fq_gemm_plan& plan, hipStream_t stream) {
    const int kblk = fq_kblk(BITS);
    // scale rows per k-block: 1, KBLK / g, or one per 32-row step when g does not divide KBLK
    const int sr = (g % kblk) == 0 ? 1 : ((kblk % g) == 0 ? kblk / g : kblk / 32);
    const int ntiles = (int)(N / FQ_NTILE);
    const int ngroups = (ntiles + NT - 1) / NT;
    const int bgroups = (ngroups + plan.gp - 1) / plan.gp;
    const int kc = kblk / 8;
    const size_t lds_act = (size_t)2 * plan.kw * kc * FQ_SK_PITCH * 16;
    const size_t lds_red = (size_t)plan.gp * plan.kw * NT * 64 * 16;
    const size_t lds = lds_act > lds_red ? lds_act : lds_red;
    const uint32_t g32 = (uint32_t)(g / 32);
    const uint32_t g32_recip = (uint32_t)((((uint64_t)1 << 32) + g32 - 1) / g32);   // unused when g32 == 1
    constexpr int STEPS = fq_kblk(BITS) / FQ_KSTEP;
    auto kern = sr == 1 ? fq_gemm_skinny_kernel<ACT, BITS, NT, DEPTH, 1, MAXW, AU>
                        : (sr == 2 ? fq_gemm_skinny_kernel<ACT, BITS, NT, DEPTH, 2, MAXW, AU>
                                   : fq_gemm_skinny_kernel<ACT, BITS, NT, DEPTH, STEPS, MAXW, AU>);
    if (lds > 65536) {
        // more than the default dynamic LDS limit: raise it for this kernel (up to the 160 KiB of a CU)
        if (lds > 160 * 1024) return FQ_ERR_UNSUPPORTED;
        static std::atomic<uint64_t> raised[3];   // per instantiation: [scale rows per k-block]
        if (raise_lds_limit((const void*)kern, raised[sr == 1 ? 0 : (sr == 2 ? 1 : 2)]) != FQ_OK) return FQ_ERR_HIP;
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
        // rows of K per k-block of this block shape (two layout blocks at a time for 8-bit codes in the
        // 128-row, 8-wave shape), and the scale rows such a k-block spans: 1, kblk / g, or one per 32-row step
        const int kblk = fq_mma_kblk(BITS, plan.mt, plan.waves, K, g);
        const bool wide = kblk != fq_kblk(BITS);
        const int sr = (g % kblk) == 0 ? 1 : ((kblk % g) == 0 ? kblk / g : kblk / 32);
        const int bm = plan.mt * 16;
        const int nblocks_n = (ntiles + plan.waves * MMA_NT - 1) / (plan.waves * MMA_NT);
        const int nblocks_m = (int)((M + bm - 1) / bm);
        // ring depth of the pipelined form per block shape (0 = two-buffer form); must match the
        // instantiations below
        const int ring = plan.mt == 8 ? (plan.waves == 8 ? 2 : 0) : (plan.mt == 4 ? FQ_RING_MT4 : FQ_RING_MT2);
        const size_t lds = (size_t)(ring ? ring + 1 : 2) * (kblk / 8) * bm * 16;
        const int64_t tiles = (int64_t)nblocks_n * nblocks_m;
        dim3 grid((unsigned)(plan.tail_tiles > 0 ? tiles - plan.tail_tiles + (int64_t)plan.tail_tiles * plan.tail_splits
                                                 : tiles * plan.splits));
        fq_group_items none;
        none.count = 0;
#define FQ_MMA_LAUNCH_SR(ACT_, A_, RS_, MT_, W_, PIPE_, SR_, KREC_)                                       \
    do {                                                                                                \
        auto kern = fq_gemm_mma_kernel<ACT_, BITS, MT_, MMA_NT, W_, SR_, false, PIPE_,                 \
                                       use_post(ACT_, BITS, MT_, SR_, PIPE_), KREC_>;                   \
        if (lds > 65536) {                                                                              \
            static std::atomic<uint64_t> raised;                                                        \
            if (raise_lds_limit((const void*)kern, raised) != FQ_OK) return FQ_ERR_HIP;                 \
        }                                                                                               \
        hipLaunchKernelGGL(kern, grid, dim3(W_ * 64), lds, stream, (const uint16_t*)(A_),               \
                           (const u32x4*)codes, (const uint16_t*)scales, (uint16_t*)C, partial, (int)M, \
                           (int)N, (int)K, g, plan.kb_per_split, plan.splits, nblocks_n, nblocks_m,     \
                           (int64_t)0, (int64_t)0, none, plan.tail_tiles, plan.tail_splits,             \
                           plan.tail_kbs, (const float*)(RS_));                                         \
    } while (0)
#define FQ_MMA_LAUNCH_ACT(ACT_, A_, RS_, MT_, W_, PIPE_)                                                \
    do {                                                                                                \
        if (sr == 1) FQ_MMA_LAUNCH_SR(ACT_, A_, RS_, MT_, W_, PIPE_, 1, 1);                             \
        else if (sr == 2) FQ_MMA_LAUNCH_SR(ACT_, A_, RS_, MT_, W_, PIPE_, 2, 1);                        \
        else if constexpr (BITS != 8) FQ_MMA_LAUNCH_SR(ACT_, A_, RS_, MT_, W_, PIPE_, 4, 1);            \
    } while (0)
// the 128-row, 8-wave shape: 8-bit codes take two layout k-blocks per k-block where K allows it
#define FQ_MMA_LAUNCH_BIG(ACT_, A_, RS_)                                                                \
    do {                                                                                                \
        if constexpr (BITS == 8) {                                                                      \
            if (wide) { /* (one scale row per k-block by construction) */                              \
                FQ_MMA_LAUNCH_SR(ACT_, A_, RS_, 8, 8, 2, 1, 2);                                         \
            } else {                                                                                    \
                FQ_MMA_LAUNCH_ACT(ACT_, A_, RS_, 8, 8, 2);                                              \
            }                                                                                           \
        } else {                                                                                        \
            FQ_MMA_LAUNCH_ACT(ACT_, A_, RS_, 8, 8, 2);                                                  \
        }                                                                                               \
    } while (0)
#define FQ_MMA_LAUNCH(MT_, W_, PIPE_) FQ_MMA_LAUNCH_ACT(ACT, A, nullptr, MT_, W_, PIPE_)
        bool launched = false;
        if constexpr (ACT == FQ_BF16) {
            if (fq_via_f16(FQ_BF16, FQ_SCALE_F16, plan, N)) {
                // bf16 activations on the fp16 matrix path: rows rewritten as binary16 first (the
                // buffers sit behind the split-K partials in the workspace)
                char* extra = (char*)workspace + fq_partial_bytes(plan, M, N);
                uint16_t* A16 = (uint16_t*)extra;
                float* rs = (float*)(extra + fq_a16_bytes(M, K));
                hipLaunchKernelGGL(fq_rows_to_f16_kernel<256>, dim3((unsigned)M), dim3(256), 0, stream,
                                   (const uint16_t*)A, (int)K, A16, rs);
                if (plan.waves == 8) FQ_MMA_LAUNCH_BIG(FQ_BF16_VIA_F16, A16, rs);
                else FQ_MMA_LAUNCH_ACT(FQ_BF16_VIA_F16, A16, rs, 8, 4, 0);
                launched = true;
            }
        }
        if constexpr (ACT == FQ_BF16_BS) {
            if (fq_via_f16(FQ_BF16, FQ_SCALE_BF16, plan, N)) {
                // the same with bfloat16 scales: their common power of two is found first
                char* extra = (char*)workspace + fq_partial_bytes(plan, M, N);
                uint16_t* A16 = (uint16_t*)extra;
                float* rs = (float*)(extra + fq_a16_bytes(M, K));
                uint32_t* parts = (uint32_t*)(rs + M + 2);
                const int64_t count = (K / g) * N;
                hipLaunchKernelGGL(fq_scale_max_kernel<256>, dim3(FQ_SCALE_PARTS), dim3(256), 0, stream,
                                   (const uint16_t*)scales, count, parts);
                hipLaunchKernelGGL(fq_scale_exp_kernel<256>, dim3(1), dim3(256), 0, stream, (const uint32_t*)parts,
                                   FQ_SCALE_PARTS, rs + M);
                hipLaunchKernelGGL(fq_rows_to_f16_kernel<256>, dim3((unsigned)M), dim3(256), 0, stream,
                                   (const uint16_t*)A, (int)K, A16, rs);
                if (plan.waves == 8) FQ_MMA_LAUNCH_BIG(FQ_BF16S_VIA_F16, A16, rs);
                else FQ_MMA_LAUNCH_ACT(FQ_BF16S_VIA_F16, A16, rs, 8, 4, 0);
                launched = true;
            }
        }
        if (launched) {
        } else if (plan.waves == 8) {
            if (plan.mt == 2) FQ_MMA_LAUNCH(2, 8, FQ_RING_MT2);
            else if (plan.mt == 4) FQ_MMA_LAUNCH(4, 8, FQ_RING_MT4);
            else FQ_MMA_LAUNCH_BIG(ACT, A, nullptr);
        } else {
            if (plan.mt == 2) FQ_MMA_LAUNCH(2, 4, FQ_RING_MT2);
            else if (plan.mt == 4) FQ_MMA_LAUNCH(4, 4, FQ_RING_MT4);
            else FQ_MMA_LAUNCH(8, 4, 0);
        }
#undef FQ_MMA_LAUNCH
#undef FQ_MMA_LAUNCH_BIG
#undef FQ_MMA_LAUNCH_ACT
#undef FQ_MMA_LAUNCH_SR
    }
    if (plan.kind == 1 && plan.tail_tiles > 0) {
        const int bm = plan.mt * 16;
        const int bn_cols = plan.waves * MMA_NT * FQ_NTILE;
        const int nblocks_n = (ntiles + plan.waves * MMA_NT - 1) / (plan.waves * MMA_NT);
        const int nblocks_m = (int)((M + bm - 1) / bm);
        hipLaunchKernelGGL(fq_reduce_tail_kernel<(ACT == FQ_F16 ? FQ_F16 : FQ_BF16)>, dim3((unsigned)plan.tail_tiles, (unsigned)plan.mt), dim3(256), 0, stream,
                           (const float*)partial, plan.tail_splits, (int)M, (int)N, nblocks_n, nblocks_m,
                           nblocks_n * nblocks_m - plan.tail_tiles, bm, bn_cols, (uint16_t*)C);
    }
    if (plan.splits > 1) {
        const int64_t MN = M * N;
        dim3 grid((unsigned)((MN / 4 + 255) / 256));
        hipLaunchKernelGGL(fq_reduce_kernel<(ACT == FQ_F16 ? FQ_F16 : FQ_BF16)>, grid, dim3(256), 0, stream, (const float*)partial,
                           plan.splits, MN, (uint16_t*)C);
    }
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}

// Grouped (per-expert) product.  Every expert's rows are cut into row tiles of 128, 64 or 32
// rows (the smallest that holds what is left), and the tiles of each size go to the kernel
// instantiated for that size: experts with few rows then stream their weights through small
// tiles instead of multiplying mostly padding.  Experts without rows produce no tile.
template <int ACT, int BITS>
int launch_grouped_typed(const void* A, const int32_t* offsets, int E, int64_t N, int64_t K,
                         const void* codes, const void* scales, int g, void* C, const hipStream_t* streams) {
    const int ntiles = (int)(N / FQ_NTILE);
    const int64_t codes_stride16 = (int64_t)(K * N * BITS / 8) / 16;
    const int64_t scales_stride = (K / g) * N;
    fq_group_items items;
    for (int mt = 8; mt >= 2; mt /= 2) {
        const int bm = mt * 16;
        // 8-wave blocks (384 columns) unless the matrix is narrow: measured 1 - 5 % faster than 4-wave
        // blocks also for the 64- and 32-row tiles (64 experts of 4096 x 16384 / 16384 x 4096)
        const int waves = (mt == 8 || ntiles >= 48) ? 8 : 4;
        const hipStream_t stream = streams[mt == 8 ? 0 : (mt == 4 ? 1 : 2)];
        const int nblocks_n = (ntiles + waves * MMA_NT - 1) / (waves * MMA_NT);
        const int ring = mt == 8 ? 2 : (mt == 4 ? FQ_RING_MT4 : FQ_RING_MT2);
        // rows of K per k-block of this tile size (8-bit codes: two layout blocks at a time in the 128-row
        // shape where K and g allow it) and the scale rows such a k-block spans
        const int kblk = fq_mma_kblk(BITS, mt, waves, K, g);
        const bool wide = kblk != fq_kblk(BITS);
        const int sr = (g % kblk) == 0 ? 1 : ((kblk % g) == 0 ? kblk / g : kblk / 32);
        const int KB = (int)(K / kblk);
        const size_t lds = (size_t)(ring ? ring + 1 : 2) * (kblk / 8) * bm * 16;
        items.count = 0;
        auto flush_items = [&]() -> int {
            if (items.count == 0) return FQ_OK;
            dim3 grid((unsigned)((int64_t)nblocks_n * items.count));
#define FQ_GROUPED_LAUNCH_SR(MT_, W_, PIPE_, SR_, KREC_)                                                 \
    do {                                                                                                \
        auto kern = fq_gemm_mma_kernel<ACT, BITS, MT_, MMA_NT, W_, SR_, true, PIPE_,                   \
                                       use_post(ACT, BITS, MT_, SR_, PIPE_), KREC_>;                    \
        if (lds > 65536) {                                                                              \
            static std::atomic<uint64_t> raised;                                                        \
            if (raise_lds_limit((const void*)kern, raised) != FQ_OK) return FQ_ERR_HIP;                 \
        }                                                                                               \
        hipLaunchKernelGGL(kern, grid, dim3(W_ * 64), lds, stream, (const uint16_t*)A,                  \
                           (const u32x4*)codes, (const uint16_t*)scales, (uint16_t*)C, (float*)nullptr, \
                           0, (int)N, (int)K, g, KB, 1, nblocks_n, items.count, codes_stride16,         \
                           scales_stride, items, 0, 1, 0, (const float*)nullptr);                       \
    } while (0)
#define FQ_GROUPED_LAUNCH(MT_, W_, PIPE_)                                                               \
    do {                                                                                                \
        if (sr == 1) FQ_GROUPED_LAUNCH_SR(MT_, W_, PIPE_, 1, 1);                                        \
        else if (sr == 2) FQ_GROUPED_LAUNCH_SR(MT_, W_, PIPE_, 2, 1);                                   \
        else if constexpr (BITS != 8) FQ_GROUPED_LAUNCH_SR(MT_, W_, PIPE_, 4, 1);                       \
    } while (0)
            if (mt == 8) {
                if constexpr (BITS == 8) {
                    if (wide) FQ_GROUPED_LAUNCH_SR(8, 8, 2, 1, 2);
                    else FQ_GROUPED_LAUNCH(8, 8, 2);
                } else {
                    FQ_GROUPED_LAUNCH(8, 8, 2);
                }
            }
            else if (mt == 4 && waves == 8) FQ_GROUPED_LAUNCH(4, 8, FQ_RING_MT4);
            else if (mt == 4) FQ_GROUPED_LAUNCH(4, 4, FQ_RING_MT4);
            else if (waves == 8) FQ_GROUPED_LAUNCH(2, 8, FQ_RING_MT2);
            else FQ_GROUPED_LAUNCH(2, 4, FQ_RING_MT2);
#undef FQ_GROUPED_LAUNCH
#undef FQ_GROUPED_LAUNCH_SR
            items.count = 0;
            return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
        };
        for (int e = 0; e < E; ++e) {
            int32_t r = offsets[e];
            while (r < offsets[e + 1]) {
                const int32_t left = offsets[e + 1] - r;
                const int tile_mt = left > 64 ? 8 : (left > 32 ? 4 : 2);
                const int32_t take = left < tile_mt * 16 ? left : tile_mt * 16;
                if (tile_mt == mt) {
                    const int i = items.count++;
                    items.row0[i] = r;
                    items.rows[i] = (int16_t)take;
                    items.expert[i] = (int16_t)e;
                    if (items.count == 256) {
                        const int st = flush_items();
                        if (st != FQ_OK) return st;
                    }
                }
                r += take;
            }
        }
        const int st = flush_items();
        if (st != FQ_OK) return st;
    }
    return FQ_OK;
}


}  // namespace fqd

// Explicitly instantiated once per (activation type, code width) in its own translation unit.
#define FQ_INSTANTIATE_GEMM(ACT, BITS)                                                                     \
    int fq_launch_typed_##ACT##_##BITS(const void* A, int64_t M, int64_t N, int64_t K, const void* codes,  \
                                       const void* scales, int g, void* C, void* workspace,                \
                                       const fq_gemm_plan& plan, hipStream_t stream) {                     \
        return fqd::launch_typed<ACT, BITS>(A, M, N, K, codes, scales, g, C, workspace, plan, stream);     \
    }                                                                                                      \
    int fq_launch_grouped_typed_##ACT##_##BITS(const void* A, const int32_t* offsets, int E, int64_t N,    \
                                               int64_t K, const void* codes, const void* scales, int g,    \
                                               void* C, const hipStream_t* streams) {                      \
        return fqd::launch_grouped_typed<ACT, BITS>(A, offsets, E, N, K, codes, scales, g, C, streams);    \
    }

#endif  // FQ_GEMM_DISPATCH_H_
