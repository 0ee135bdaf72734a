// Fused dequantise-and-multiply kernels for gfx950 (section 4.1, "GPU kernel
// implementations": int4/int8 weights with a matrix of scales, fp16/bf16 activations,
// floating-point matrix-core math, output in the activation type; 3-bit codes, which the
// paper evaluates for accuracy only, run through the same kernels).
//
// Orientation: every product is computed as 16x16 tiles of C^T with
// v_mfma_f32_16x16x32_{f16,bf16}.  The WEIGHTS are the first MFMA operand (its 16 rows are
// 16 output columns n), the ACTIVATIONS the second (its 16 columns are 16 rows m of A).
// A lane's record of the packed layout (16 bytes; 12 for 3-bit codes) is, after the integer->float step, directly
// its slice of the first operand: weights never pass through LDS.  The result tile leaves
// lane l with C[m = l % 16][n = 4 (l / 16) + 0..3], i.e. four consecutive columns of one row.
//
// Numerics, small-M kernel and the post-scaled form of the large-M kernel: the integer codes are
// converted EXACTLY to the activation type (bf16 carries them with a constant offset that is
// removed in binary32), multiplied on the matrix cores with binary32 accumulation over one scale
// group (or one k-block), and the group's scale is applied to that partial sum in binary32;
// nothing is rounded to 16 bits before the final store.  The pre-scaled form of the large-M kernel
// rounds q * s once to the activation type before the MFMA (the paper's order).
//
// (device code; included by the per-type translation units through fq_gemm_dispatch.h)
#ifndef FQ_GEMM_KERNELS_H_
#define FQ_GEMM_KERNELS_H_

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "fq_internal.h"
#include "fq_layout.h"

namespace fqk {

// Third value of the ACT template argument next to FQ_F16 / FQ_BF16: bfloat16 activations whose
// scale matrix holds bfloat16 values (section 4.1, "GPU kernel implementations": scales of the
// activation's data type).  It behaves as FQ_BF16 everywhere except where a scale is widened.
#define FQ_BF16_BS 2
// Fourth value: bfloat16 activations and output, computed on the fp16 matrix path.  A small kernel
// first rewrites the activation rows as binary16, each row divided by a power of two that brings its
// largest element into [2^14, 2^15) (exact for every element within 2^-29 of the row's largest; what
// lies further below loses low bits or vanishes, 2^-25 of the row's scale at most); the weights are
// dequantised to binary16 (three more significand bits than bfloat16), and the epilogue multiplies the
// binary32 sums by the row's power of two before rounding to bfloat16.  The fp16 conversion of the
// codes is packed (13 vector instructions per 8 weights against 23 for bf16), which is what the large-M
// loop is short of.  Used by the 128-row shapes only.
#define FQ_BF16_VIA_F16 3
// Fifth value: the same path for bfloat16 SCALES (FQ_BF16_BS computed with fp16 MFMAs).  A bfloat16 scale has
// eight significant bits but binary32's exponent range, so the scales are first multiplied by 2^-E, E the
// exponent of the largest scale of the matrix (found by fq_scale_maxexp_kernel): they then lie in (0, 2) and
// convert to binary16 exactly unless they are more than 2^14 times smaller than the largest one (those lose
// low bits or vanish: their weights are below 2^-14 of the matrix's widest group).  q * s * 2^-E is rounded
// once to binary16 (at most 4 + 8 significant bits: usually exact), and the epilogue multiplies by 2^E.
#define FQ_BF16S_VIA_F16 4

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename T, typename F>
__device__ inline T bitcast(const F& f) {
    static_assert(sizeof(T) == sizeof(F), "size mismatch");
    return __builtin_bit_cast(T, f);
}

// A wave-uniform pointer pinned in scalar registers and hidden from the optimiser: an address formed as
// (this) + (32-bit lane offset) is then taken by a global load as scalar base + vector offset; left
// alone, the compiler folds the lane offset into a 64-bit vector base outside the loop and adds the
// loop-dependent uniform part with vector instructions at every load.
// (The round trip through integers drops the address space, hence the explicit global one.)
#define FQ_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ inline const FQ_GLOBAL T* scalar_ptr(const T* p) {
    uint32_t lo = (uint32_t)(uintptr_t)p, hi = (uint32_t)((uintptr_t)p >> 32);
    asm volatile("" : "+s"(lo), "+s"(hi));
    return reinterpret_cast<const FQ_GLOBAL T*>(((uintptr_t)hi << 32) | (uintptr_t)lo);
}

// One lane record of packed codes: 16 bytes, or 12 bytes (three dwords, the fourth left zero) for
// 3-bit codes.  Either way a single vector load.
template <int BITS, bool NONTEMPORAL, typename P>   // P: const char* in the generic or the global address space
__device__ inline u32x4 load_rec(P p) {
    if constexpr (BITS == 3) {
        // three dwords with 4-byte alignment (one 12-byte load)
        typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
        typedef u32x3 __attribute__((aligned(4))) u32x3a;
        typedef typename std::conditional<std::is_same<P, const char*>::value, const u32x3a*, const FQ_GLOBAL u32x3a*>::type R;
        const u32x3 v = *reinterpret_cast<R>(p);
        u32x4 r = {v[0], v[1], v[2], 0u};
        return r;
    } else {
        typedef typename std::conditional<std::is_same<P, const char*>::value, const u32x4*, const FQ_GLOBAL u32x4*>::type R;
        if constexpr (NONTEMPORAL) {
            return __builtin_nontemporal_load(reinterpret_cast<R>(p));
        } else {
            return *reinterpret_cast<R>(p);
        }
    }
}

template <int ACT>
__device__ inline f32x4 mfma16x16x32(const u32x4& w, const u32x4& a, const f32x4& c) {
    if constexpr (ACT == FQ_F16 || ACT == FQ_BF16_VIA_F16 || ACT == FQ_BF16S_VIA_F16) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(bitcast<f16x8>(w), bitcast<f16x8>(a), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(bitcast<bf16x8>(w), bitcast<bf16x8>(a), c, 0, 0, 0);
    }
}

// ------------------------------------------------------------------------------------------
// Integer code -> matrix-core operand.  The result holds (q + OFFSET) exactly.
//   fp16: the stored nibble/byte u is OR-ed into the mantissa of 1024.0 (0x6400), giving
//         1024 + u (or 1024 + 16 u for the nibble that sits four bits higher), and one packed
//         fp16 add / fma removes 1024 and the storage bias exactly:  OFFSET = 0.
//   bf16: there is no packed bf16 arithmetic on gfx950, so the operand keeps a bias:
//         4-bit: 0x4300 | u = 128 + u      -> OFFSET = 136 (= 128 + 8)
//         8-bit: float(u) truncated to bf16 is exact for u <= 255 -> OFFSET = 128
//         The bias is removed after the MFMA with the row sums of A over the same k-range,
//         which an extra MFMA against an all-ones operand provides.
// ------------------------------------------------------------------------------------------
// (x & mask) | magic in one v_and_or_b32.  gfx9 VALU instructions can read only one
// scalar/literal operand, so the magic constant is pinned in a vector register (the empty
// asm hides its value from the constant folder); otherwise the compiler splits the
// operation into v_and_b32 + v_or_b32.
__device__ inline uint32_t vgpr_const(uint32_t c) {
    asm volatile("" : "+v"(c));
    return c;
}
__device__ inline uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic_v) { return (x & mask) | magic_v; }

template <int ACT, int BITS>
struct Dequant;

// The 32-bit word that holds the eight stored values of k-step T of a sub-byte record, one per
// nibble.  4-bit: dword T as it is.  3-bit: dwords 0..2 as they are (the values sit in the low three
// bits of the nibbles; the fourth bit belongs to step 3 and is dropped by the conversion masks), and
// step 3 is gathered from those fourth bits.
template <int SB, int T>
__device__ inline uint32_t code_word(const u32x4& rec) {
    if constexpr (SB == 3 && T == 3) {
        return ((rec[0] >> 3) & 0x11111111u) | ((rec[1] >> 2) & 0x22222222u) | ((rec[2] >> 1) & 0x44444444u);
    } else {
        return rec[T];
    }
}

// SB-bit codes (SB = 3 or 4), stored value u = q + 2^(SB-1) in the low SB bits of a nibble
template <int SB>
struct DequantF16Sub {
    static constexpr float OFFSET = 0.0f;
    static constexpr uint32_t MLO = SB == 4 ? 0x000f000fu : 0x00070007u;
    static constexpr float BIAS = SB == 4 ? 8.0f : 4.0f;
    static __device__ inline uint32_t init() { return vgpr_const(0x64006400u); }
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec, uint32_t MAGIC) {
        const uint32_t w = code_word<SB, T>(rec);
        const uint32_t w8 = w >> 8;
        const f16x2 lo0 = bitcast<f16x2>(and_or(w, MLO, MAGIC));
        const f16x2 hi0 = bitcast<f16x2>(and_or(w, MLO << 4, MAGIC));
        const f16x2 lo1 = bitcast<f16x2>(and_or(w8, MLO, MAGIC));
        const f16x2 hi1 = bitcast<f16x2>(and_or(w8, MLO << 4, MAGIC));
        const f16x2 sub = {(_Float16)(1024.0f + BIAS), (_Float16)(1024.0f + BIAS)};
        const f16x2 sc = {(_Float16)0.0625f, (_Float16)0.0625f};
        const f16x2 off = {(_Float16)(-64.0f - BIAS), (_Float16)(-64.0f - BIAS)};
        u32x4 r;
        r[0] = bitcast<uint32_t>(lo0 - sub);                                 // elements 0,1
        r[1] = bitcast<uint32_t>(__builtin_elementwise_fma(hi0, sc, off));   // elements 2,3
        r[2] = bitcast<uint32_t>(lo1 - sub);                                 // elements 4,5
        r[3] = bitcast<uint32_t>(__builtin_elementwise_fma(hi1, sc, off));   // elements 6,7
        return r;
    }
};
template <>
struct Dequant<FQ_F16, 4> : DequantF16Sub<4> {};
template <>
struct Dequant<FQ_F16, 3> : DequantF16Sub<3> {};

template <>
struct Dequant<FQ_F16, 8> {
    static constexpr float OFFSET = 0.0f;
    static __device__ inline uint32_t init() { return 0x64646464u; }
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec, uint32_t MAGIC) {
        const uint32_t w0 = rec[2 * T], w1 = rec[2 * T + 1];
        const f16x2 sub = {(_Float16)1152.0f, (_Float16)1152.0f};   // 1024 + 128
        u32x4 r;
        r[0] = bitcast<uint32_t>(bitcast<f16x2>(__builtin_amdgcn_perm(MAGIC, w0, 0x04010400u)) - sub);
        r[1] = bitcast<uint32_t>(bitcast<f16x2>(__builtin_amdgcn_perm(MAGIC, w0, 0x04030402u)) - sub);
        r[2] = bitcast<uint32_t>(bitcast<f16x2>(__builtin_amdgcn_perm(MAGIC, w1, 0x04010400u)) - sub);
        r[3] = bitcast<uint32_t>(bitcast<f16x2>(__builtin_amdgcn_perm(MAGIC, w1, 0x04030402u)) - sub);
        return r;
    }
};

template <int SB>
struct DequantBF16Sub {
    static constexpr float OFFSET = SB == 4 ? 136.0f : 132.0f;     // 128 + the storage bias
    static constexpr uint32_t MLO = SB == 4 ? 0x000f000fu : 0x00070007u;
    static __device__ inline uint32_t init() { return vgpr_const(0x43004300u); }
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec, uint32_t MAGIC) {
        const uint32_t w = code_word<SB, T>(rec);
        u32x4 r;
        r[0] = and_or(w, MLO, MAGIC);
        r[1] = and_or(w >> 4, MLO, MAGIC);
        r[2] = and_or(w >> 8, MLO, MAGIC);
        r[3] = and_or(w >> 12, MLO, MAGIC);
        return r;
    }
};
template <>
struct Dequant<FQ_BF16, 4> : DequantBF16Sub<4> {};
template <>
struct Dequant<FQ_BF16, 3> : DequantBF16Sub<3> {};

template <>
struct Dequant<FQ_BF16, 8> {
    static constexpr float OFFSET = 128.0f;
    static __device__ inline uint32_t init() { return 0u; }
    static __device__ inline uint32_t pair(uint32_t w, int lo_byte) {
        const float f0 = (float)((w >> (8 * lo_byte)) & 0xffu);
        const float f1 = (float)((w >> (8 * lo_byte + 8)) & 0xffu);
        // upper halves of the two binary32 values (exact: at most 8 significant bits)
        return __builtin_amdgcn_perm(bitcast<uint32_t>(f1), bitcast<uint32_t>(f0), 0x07060302u);
    }
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec, uint32_t MAGIC) {
        const uint32_t w0 = rec[2 * T], w1 = rec[2 * T + 1];
        u32x4 r;
        r[0] = pair(w0, 0);
        r[1] = pair(w0, 2);
        r[2] = pair(w1, 0);
        r[3] = pair(w1, 2);
        return r;
    }
};

template <int BITS>
struct Dequant<FQ_BF16_BS, BITS> : Dequant<FQ_BF16, BITS> {};
template <int BITS>
struct Dequant<FQ_BF16_VIA_F16, BITS> : Dequant<FQ_F16, BITS> {};
template <int BITS>
struct Dequant<FQ_BF16S_VIA_F16, BITS> : Dequant<FQ_F16, BITS> {};

template <int ACT>
__device__ inline u32x4 ones_operand() {
    const uint32_t one2 = ACT == FQ_F16 ? 0x3c003c00u : 0x3f803f80u;
    u32x4 r = {one2, one2, one2, one2};
    return r;
}

template <int ACT>
__device__ inline u32x2 pack4(const f32x4& v) {
    u32x2 r;
    if constexpr (ACT == FQ_F16) {
        const f16x2 a = {(_Float16)v[0], (_Float16)v[1]};
        const f16x2 b = {(_Float16)v[2], (_Float16)v[3]};
        r[0] = bitcast<uint32_t>(a);
        r[1] = bitcast<uint32_t>(b);
    } else {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const bf16x2 a = {(__bf16)v[0], (__bf16)v[1]};
        const bf16x2 b = {(__bf16)v[2], (__bf16)v[3]};
        r[0] = bitcast<uint32_t>(a);
        r[1] = bitcast<uint32_t>(b);
    }
    return r;
}

// acc += s * (p - OFFSET * rowsum)
template <int ACT, int BITS>
__device__ inline void flush(f32x4& acc, const f32x4& p, const f32x4& s, float rowsum) {
    constexpr float OFF = Dequant<ACT, BITS>::OFFSET;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float d = p[i];
        if constexpr (OFF != 0.0f) d = __builtin_fmaf(-OFF, rowsum, d);
        acc[i] = __builtin_fmaf(s[i], d, acc[i]);
    }
}

// ==========================================================================================
// Small-M kernel (M <= 16): the decode case, bound by the HBM read of the weights
// (section 2.1, "Large weights with small activations").
//
// Block = GP column groups x KW k-workers (run-time values, GP * KW <= MAXW waves), one block
// per compute unit and all blocks resident at once: a wave's loop is latency-bound, so a
// second, partly filled round of blocks would cost as much as the first.  Wave (gi, kw) owns
// NT column tiles and, in iteration `it`, k-block (sb * KW + kw) of super-block sb.
//  - Weights and scales stream through a DEPTH-deep REGISTER ring per wave (NT KiB per stage);
//    they never touch LDS.
//  - The activation slice of a super-block (M rows x KW k-blocks) is fetched ONCE per block by
//    a cooperative, coalesced load, DEPTH iterations ahead (two registers per lane in the same
//    ring, so its age in the in-order memory queue equals that of the weights consumed with
//    it), written to one of two LDS buffers and read back as MFMA fragments.  Fetching it per
//    wave from L1/L2 instead costs four more vector loads per k-block and wave, and those, not
//    HBM, were what limited the rate.
//  - One barrier per iteration; the steady-state loop has no conditionals, so the memory
//    counter waits only for the stage about to be consumed.
//  - The KW partial results of a column group are added through LDS (fixed order); if the grid
//    also splits K (grid_splits > 1) block sums go to a binary32 partial buffer.
// SR = scale rows per k-block: 1 when the group size is a multiple of KBLK, else KBLK / g, or one per
// 32-row k-step when g does not divide KBLK.
// ==========================================================================================
// AU = activation units (16 B) a lane fetches per super-block: M * KC <= AU * 64 * GP.
template <int BITS, int NT, int SR, int AU_>
struct SkinnyStage {
    static constexpr int STEPS = fq_kblk(BITS) / FQ_KSTEP;
    static constexpr int AU = AU_;
    u32x4 wq[NT];
    // four scales (output columns 4j .. 4j+3) of one scale row.  SR > 1: the lane holds the row of
    // k-step (lane % STEPS), so each quad of lanes holds all the rows of the k-block and a
    // quad broadcast hands every lane the row of the step at hand: one load per tile and k-block
    // instead of one per step.
    u32x2 sc[NT];
    u32x4 areg[AU];
};

// four stored scales -> binary32
template <int ACT>
__device__ inline f32x4 scales4(const u32x2& v) {
    if constexpr (ACT == FQ_BF16_BS) {
        f32x4 r = {bitcast<float>(v[0] << 16), bitcast<float>(v[0] & 0xffff0000u),
                   bitcast<float>(v[1] << 16), bitcast<float>(v[1] & 0xffff0000u)};
        return r;
    } else {
        const f16x2 a = bitcast<f16x2>(v[0]);
        const f16x2 b = bitcast<f16x2>(v[1]);
        f32x4 r = {(float)a[0], (float)a[1], (float)b[0], (float)b[1]};
        return r;
    }
}

// value of lane (4 * (lane / 4) + T) for every lane of the quad
template <int T>
__device__ inline u32x2 quad_bcast(const u32x2& v) {
    u32x2 r;
    r[0] = (uint32_t)__builtin_amdgcn_mov_dpp((int)v[0], T * 0x55, 0xf, 0xf, true);
    r[1] = (uint32_t)__builtin_amdgcn_mov_dpp((int)v[1], T * 0x55, 0xf, 0xf, true);
    return r;
}

// acc[nt] += (this wave's k-block of the stage) x (activation fragments af[0..STEPS)).
// The k-steps of one scale row (STEPS / SR of them) accumulate in p, which is then folded into acc with
// that row's scales.
template <int ACT, int BITS, int NT, int SR, int AU>
__device__ inline void skinny_block(const SkinnyStage<BITS, NT, SR, AU>& sl,
                                    const u32x4 (&af)[SkinnyStage<BITS, NT, SR, AU>::STEPS], uint32_t magic,
                                    f32x4 (&acc)[NT]) {
    constexpr int STEPS = SkinnyStage<BITS, NT, SR, AU>::STEPS;
    constexpr int GSTEPS = STEPS / SR;
    static_assert(SR >= 1 && STEPS % SR == 0, "");
    constexpr float OFF = Dequant<ACT, BITS>::OFFSET;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < SR; ++r) {
        f32x4 p[NT];
        f32x4 psa = zero;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) p[nt] = zero;
#pragma unroll
        for (int u = 0; u < GSTEPS; ++u) {
            const int t = r * GSTEPS + u;
            const u32x4 a = af[t];
            if constexpr (OFF != 0.0f) psa = mfma16x16x32<ACT>(ones_operand<ACT>(), a, psa);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                u32x4 w;
                if (t == 0) w = Dequant<ACT, BITS>::template run<0>(sl.wq[nt], magic);
                if (t == 1) w = Dequant<ACT, BITS>::template run<1>(sl.wq[nt], magic);
                if (STEPS > 2 && t == 2) w = Dequant<ACT, BITS>::template run<2 % STEPS>(sl.wq[nt], magic);
                if (STEPS > 2 && t == 3) w = Dequant<ACT, BITS>::template run<3 % STEPS>(sl.wq[nt], magic);
                p[nt] = mfma16x16x32<ACT>(w, a, p[nt]);
            }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            u32x2 sq = sl.sc[nt];
            if constexpr (SR > 1) {
                // the lane of the quad that fetched the row of this scale row's first k-step
                const int t0 = r * GSTEPS;
                if (t0 == 0) sq = quad_bcast<0>(sl.sc[nt]);
                if (t0 == 1) sq = quad_bcast<1>(sl.sc[nt]);
                if (STEPS > 2 && t0 == 2) sq = quad_bcast<2 % STEPS>(sl.sc[nt]);
                if (STEPS > 2 && t0 == 3) sq = quad_bcast<3 % STEPS>(sl.sc[nt]);
            }
            flush<ACT, BITS>(acc[nt], p[nt], scales4<ACT>(sq), psa[0]);
        }
    }
}

// LDS row pitch of the activation buffer in 16-byte units: 16 rows + 1 pad, so that both the
// fragment reads (16 lanes = 16 rows of one unit column) and the staging writes (consecutive
// lanes = consecutive unit columns of one row) spread over the banks.
#define FQ_SK_PITCH 17

template <int ACT, int BITS, int NT, int DEPTH, int SR, int MAXW, int AU>
__global__ __launch_bounds__(MAXW * 64) void fq_gemm_skinny_kernel(
    const uint16_t* __restrict__ A, const u32x4* __restrict__ codes, const uint16_t* __restrict__ scales,
    uint16_t* __restrict__ C, float* __restrict__ partial, int M, int N, int K, uint32_t g32,
    uint32_t g32_recip, int gp, int kw_n, int grid_splits) {
    constexpr int KBLK = fq_kblk(BITS);
    constexpr int STEPS = KBLK / FQ_KSTEP;
    constexpr int KC = KBLK / 8;                    // 16-byte activation units per row and k-block
    typedef SkinnyStage<BITS, NT, SR, AU> Stage;
    extern __shared__ u32x4 lds[];   // two activation buffers [kw_n * KC][FQ_SK_PITCH]; later the reduction

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int gi = wave / kw_n;
    const int kw = wave - gi * kw_n;
    const int ntiles = N / FQ_NTILE;
    const int ngroups = (ntiles + NT - 1) / NT;
    const int bgroups = (ngroups + gp - 1) / gp;      // blocks per grid split
    const int bx = blockIdx.x % bgroups;
    const int gsplit = blockIdx.x / bgroups;          // < grid_splits
    const int ng = bx * gp + gi;
    const bool gvalid = ng < ngroups;
    const int KB = K / KBLK;
    const int SB = (KB + kw_n - 1) / kw_n;            // super-blocks of kw_n k-blocks
    const int n_it = gsplit < SB ? (SB - gsplit + grid_splits - 1) / grid_splits : 0;   // block-uniform
    const int64_t kb_stride = (int64_t)ntiles * 64;   // records between consecutive k-blocks of a tile
    const int m = lane & 15, j = lane >> 4;
    const uint32_t magic = Dequant<ACT, BITS>::init();
    const int abuf_units = kw_n * KC * FQ_SK_PITCH;

    // Wave-uniform bases (scalar registers) plus one per-lane offset each.
    constexpr int RB = fq_rec_bytes(BITS);
    const char* wbase[NT];
    const uint16_t* sbase[NT];
    bool tvalid[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tile = ng * NT + nt;
        tvalid[nt] = gvalid && tile < ntiles;
        const int tc = tvalid[nt] ? tile : 0;
        wbase[nt] = reinterpret_cast<const char*>(codes) + fq_rec(tc, 0, ntiles, 0) * RB;
        sbase[nt] = scales + tc * FQ_NTILE;
    }
    const uint32_t s_off = (uint32_t)j * 4u;

    // Cooperative activation fetch: unit u = tid + r * nthreads covers row u / upr, unit column
    // u % upr of the super-block (upr = kw_n * KC units of 8 values per row).
    const int upr = kw_n * KC;
    int a_row[AU], a_col[AU];
#pragma unroll
    for (int r = 0; r < AU; ++r) {
        const int u = tid + r * nthreads;
        a_row[r] = u / upr;
        a_col[r] = u - a_row[r] * upr;
    }

    f32x4 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    auto load_act = [&](u32x4 (&areg)[AU], int it) {
        const int64_t k0 = (int64_t)(gsplit + it * grid_splits) * kw_n * KBLK;
#pragma unroll
        for (int r = 0; r < AU; ++r) {
            int64_t k = k0 + a_col[r] * 8;
            k = k < K ? k : K - 8;                       // past the end (tail super-block): never multiplied
            areg[r] = a_row[r] < M ? *reinterpret_cast<const u32x4*>(A + (int64_t)a_row[r] * K + k) : zero4;
        }
    };
    auto store_act = [&](const u32x4 (&areg)[AU], int buf) {
#pragma unroll
        for (int r = 0; r < AU; ++r)
            if (a_row[r] < 16) lds[buf * abuf_units + a_col[r] * FQ_SK_PITCH + a_row[r]] = areg[r];
    };
    // stage `it`: this wave's weights and scales for iteration it, and the lane's share of the
    // activations of iteration it + 1
    auto load_stage = [&](Stage& sl, int it) {
        int kb = (gsplit + it * grid_splits) * kw_n + kw;
        kb = kb < KB ? kb : KB - 1;                      // tail super-block: idle workers re-read the last block
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) sl.wq[nt] = load_rec<BITS, true>(wbase[nt] + ((int64_t)kb * kb_stride + lane) * RB);
        {
            // scale row of a 32-row k-step: an exact division by g / 32 done as a multiplication by
            // its rounded-up reciprocal (valid while the step index < 2^32 / (g/32)).  SR > 1: the
            // lane fetches the row of step (lane % STEPS) of the k-block.
            const uint32_t step = (uint32_t)kb * STEPS + (SR > 1 ? (uint32_t)(lane & (STEPS - 1)) : 0u);
            const uint32_t row = g32 == 1 ? step : __umulhi(step, g32_recip);
            const int64_t srow = (int64_t)row * N;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                sl.sc[nt] = *reinterpret_cast<const u32x2*>(sbase[nt] + srow + s_off);
        }
        load_act(sl.areg, it + 1);
    };
    // one iteration: publish the next activations, read this iteration's fragments, multiply
    auto iterate = [&](const Stage& sl, int it) {
        store_act(sl.areg, (it + 1) & 1);
        const int kb = (gsplit + it * grid_splits) * kw_n + kw;
        u32x4 af[STEPS];
        const u32x4* abuf = lds + (it & 1) * abuf_units + (kw * KC + j) * FQ_SK_PITCH + m;
#pragma unroll
        for (int t = 0; t < STEPS; ++t) af[t] = abuf[t * 4 * FQ_SK_PITCH];
        if (gvalid && kb < KB) skinny_block<ACT, BITS, NT, SR, AU>(sl, af, magic, acc);
    };

    if (n_it > 0) {
        {   // activations of iteration 0
            u32x4 a0[AU];
            load_act(a0, 0);
            store_act(a0, 0);
        }
        Stage ring[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (d < n_it) load_stage(ring[d], d);
        __syncthreads();
        int it = 0;
        for (; it + 2 * DEPTH <= n_it; it += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                iterate(ring[d], it + d);
                load_stage(ring[d], it + d + DEPTH);
                __syncthreads();
            }
        }
        // drain: at most 2 * DEPTH - 1 iterations are left, the first min(DEPTH, left) already loaded
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (it + d < n_it) {
                iterate(ring[d], it + d);
                if (it + d + DEPTH < n_it) load_stage(ring[d], it + d + DEPTH);
                __syncthreads();
            }
        }
#pragma unroll
        for (int d = 0; d < DEPTH - 1; ++d) {
            if (it + d + DEPTH < n_it) {
                iterate(ring[d], it + d + DEPTH);
                __syncthreads();
            }
        }
    }

    // Combine the k-workers of each column group in fixed order (worker 0 + worker 1 + worker 2 ...).  Every
    // wave parks its sums in LDS and the block's threads share the NT * 64 result quads of every group, so that
    // each thread adds kw_n independent values (one wave adding all of them one after the other spent a
    // dependent LDS round trip per worker and tile: 2.6 us of the 17 us the 12288 x 12288 layer takes).
    auto store_quad = [&](const f32x4& v, int group, int nt, int ln) {
        const int mq = ln & 15, jq = ln >> 4;
        const int tile = group * NT + nt;
        if (mq >= M || group >= ngroups || tile >= ntiles) return;
        const int64_t n = (int64_t)tile * FQ_NTILE + jq * 4;
        if (grid_splits == 1) {
            *reinterpret_cast<u32x2*>(C + (int64_t)mq * N + n) = pack4<ACT>(v);
        } else {
            *reinterpret_cast<f32x4*>(partial + ((int64_t)gsplit * M + mq) * N + n) = v;
        }
    };
    if (kw_n == 1) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) store_quad(acc[nt], ng, nt, lane);
        return;
    }
    f32x4* red = reinterpret_cast<f32x4*>(lds);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) red[(wave * NT + nt) * 64 + lane] = acc[nt];
    __syncthreads();
    const int nquads = gp * NT * 64;
    for (int q = tid; q < nquads; q += nthreads) {
        const int gq = q / (NT * 64);            // column group of the block
        const int r = q - gq * (NT * 64);        // nt * 64 + lane inside the group
        const f32x4* src = red + (int64_t)gq * kw_n * NT * 64 + r;   // worker w: + w * NT * 64
        f32x4 v = src[0];
#pragma unroll 4
        for (int w = 1; w < kw_n; ++w) {
            const f32x4 o = src[w * NT * 64];
            v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
        }
        store_quad(v, bx * gp + gq, r >> 6, r & 63);
    }
}

// Sum of split-K partials, fixed order, then conversion to the activation type.
template <int ACT>
__global__ __launch_bounds__(256) void fq_reduce_kernel(const float* __restrict__ partial, int splits,
                                                        int64_t MN, uint16_t* __restrict__ C) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= MN) return;
    f32x4 v = *reinterpret_cast<const f32x4*>(partial + i);
    for (int s = 1; s < splits; ++s) {
        const f32x4 o = *reinterpret_cast<const f32x4*>(partial + (int64_t)s * MN + i);
        v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
    }
    *reinterpret_cast<u32x2*>(C + i) = pack4<ACT>(v);
}

// One row tile of a grouped (per-expert) product: rows [row0, row0 + rows) of the stacked
// activations belong to expert `expert`.  Passed by value in the kernel arguments.
struct fq_group_items {
    int count;
    int32_t row0[256];
    int16_t rows[256];
    int16_t expert[256];
};

// ==========================================================================================
// Large-M kernel (prefill): pre-scaled weights, one accumulator set.
//
// Section 4.1 reports that in compute-bound cases the integer->float conversion, not the
// matrix-core math, limits such kernels.  Here every weight record is converted AND scaled
// exactly once per block (by the one wave that owns its columns) and then reused for all
// BM = 16 MT rows of the block straight from registers; the conversion cost per MFMA is
// therefore 1/MT of a fragment conversion.  Scaling before the MFMA (the order section 4.1
// describes: weights are brought to the activation type, then multiplied) keeps a single set
// of accumulators, which is what allows MT = 8.
//   fp16: q (exact) * s rounded once to fp16          (relative error <= 2^-11 per weight)
//   bf16: fma(u, s, -bias * s) in binary32 = q * s exactly, rounded once to bf16 (<= 2^-9)
// Block = WAVES waves, all sharing one activation tile (BM x KBLK) staged through LDS (two
// or three buffers); wave w owns column tiles [(bx * WAVES + w) * NT, +NT).
// With GROUPED, row tile i of the grid is items.row0/rows/expert[i] and the weights of expert e
// start e * codes_stride16 records / e * scales_stride scales into the buffers.
// ==========================================================================================
template <int ACT, int BITS>
struct DequantScaled;

template <int SB>
struct DequantScaledF16Sub {
    // s2 = (s, s) as packed fp16
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec, uint32_t MAGIC, uint32_t s2) {
        const u32x4 q = Dequant<FQ_F16, SB>::template run<T>(rec, MAGIC);
        const f16x2 s = bitcast<f16x2>(s2);
        u32x4 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = bitcast<uint32_t>(bitcast<f16x2>(q[i]) * s);
        return r;
    }
};
template <>
struct DequantScaled<FQ_F16, 4> : DequantScaledF16Sub<4> {};
template <>
struct DequantScaled<FQ_F16, 3> : DequantScaledF16Sub<3> {};

template <>
struct DequantScaled<FQ_F16, 8> {
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec, uint32_t MAGIC, uint32_t s2) {
        const u32x4 q = Dequant<FQ_F16, 8>::template run<T>(rec, MAGIC);
        const f16x2 s = bitcast<f16x2>(s2);
        u32x4 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = bitcast<uint32_t>(bitcast<f16x2>(q[i]) * s);
        return r;
    }
};

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 v = {(__bf16)lo, (__bf16)hi};
    return bitcast<uint32_t>(v);
}

template <int SB>
struct DequantScaledBF16Sub {
    // s2 = binary32 bits of the scale
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec, uint32_t, uint32_t s2) {
        const uint32_t w = code_word<SB, T>(rec);
        const float s = bitcast<float>(s2);
        const float b = (SB == 4 ? -8.0f : -4.0f) * s;
        constexpr uint32_t M = SB == 4 ? 0x0f0f0f0fu : 0x07070707u;
        uint32_t lo = w & M;          // nibbles 0,2,4,6 = elements 0,4,1,5
        uint32_t hi = (w >> 4) & M;   // nibbles 1,3,5,7 = elements 2,6,3,7
        // opaque to the optimiser: byte k of lo / hi then converts with one v_cvt_f32_ubyte<k>
        // instead of a bit-field extract plus a conversion
        asm("" : "+v"(lo));
        asm("" : "+v"(hi));
        auto f = [&](uint32_t x, int byte) { return __builtin_fmaf((float)((x >> (8 * byte)) & 0xffu), s, b); };
        u32x4 r;
        r[0] = pack_bf16x2(f(lo, 0), f(lo, 2));
        r[1] = pack_bf16x2(f(hi, 0), f(hi, 2));
        r[2] = pack_bf16x2(f(lo, 1), f(lo, 3));
        r[3] = pack_bf16x2(f(hi, 1), f(hi, 3));
        return r;
    }
};
template <>
struct DequantScaled<FQ_BF16, 4> : DequantScaledBF16Sub<4> {};
template <>
struct DequantScaled<FQ_BF16, 3> : DequantScaledBF16Sub<3> {};

template <>
struct DequantScaled<FQ_BF16, 8> {
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec, uint32_t, uint32_t s2) {
        const uint32_t w0 = rec[2 * T], w1 = rec[2 * T + 1];
        const float s = bitcast<float>(s2);
        const float b = -128.0f * s;
        auto f = [&](uint32_t x, int byte) { return __builtin_fmaf((float)((x >> (8 * byte)) & 0xffu), s, b); };
        u32x4 r;
        r[0] = pack_bf16x2(f(w0, 0), f(w0, 1));
        r[1] = pack_bf16x2(f(w0, 2), f(w0, 3));
        r[2] = pack_bf16x2(f(w1, 0), f(w1, 1));
        r[3] = pack_bf16x2(f(w1, 2), f(w1, 3));
        return r;
    }
};

template <int BITS>
struct DequantScaled<FQ_BF16_BS, BITS> : DequantScaled<FQ_BF16, BITS> {};
template <int BITS>
struct DequantScaled<FQ_BF16_VIA_F16, BITS> : DequantScaled<FQ_F16, BITS> {};
template <int BITS>
struct DequantScaled<FQ_BF16S_VIA_F16, BITS> : DequantScaled<FQ_F16, BITS> {};

// stored scale (16 bits) -> the form DequantScaled wants (sshift: 2^-E for FQ_BF16S_VIA_F16, unused otherwise)
template <int ACT>
__device__ inline uint32_t scale_operand(uint16_t h, float sshift) {
    if constexpr (ACT == FQ_F16 || ACT == FQ_BF16_VIA_F16) {
        return (uint32_t)h | ((uint32_t)h << 16);
    } else if constexpr (ACT == FQ_BF16S_VIA_F16) {
        const _Float16 s = (_Float16)(bitcast<float>((uint32_t)h << 16) * sshift);
        const uint32_t b = (uint32_t)bitcast<uint16_t>(s);
        return b | (b << 16);
    } else if constexpr (ACT == FQ_BF16_BS) {
        return (uint32_t)h << 16;
    } else {
        return bitcast<uint32_t>((float)bitcast<_Float16>(h));
    }
}

// Logical tile -> (column block, row block).  Logical tiles walk panels of PW column blocks x all
// row blocks, so that the blocks resident on an XCD at one time share activation rows and weight
// columns in its L2.
__device__ inline void fq_tile_of(int L, int nblocks_n, int nblocks_m, int& bn, int& bm) {
    const int PW = nblocks_n < 4 ? nblocks_n : 4;
    const int panel = L / (PW * nblocks_m);
    const int within = L - panel * PW * nblocks_m;
    const int pw_here = min(PW, nblocks_n - panel * PW);
    bm = within / pw_here;
    bn = panel * PW + within - bm * pw_here;
}

// Sum of the partial tiles of the last `tail_tiles` logical tiles (fixed order); block (x, y) takes rows
// [16 y, 16 y + 16) of tile x.
template <int ACT>
__global__ __launch_bounds__(256) void fq_reduce_tail_kernel(const float* __restrict__ partial, int tail_splits,
                                                             int M, int N, int nblocks_n, int nblocks_m,
                                                             int head, int bm_rows, int bn_cols,
                                                             uint16_t* __restrict__ C) {
    int bn, bm;
    fq_tile_of(head + blockIdx.x, nblocks_n, nblocks_m, bn, bm);
    const int row0 = bm * bm_rows + 16 * blockIdx.y, col0 = bn * bn_cols;
    const int rows = min(16, M - row0), cols = min(bn_cols, N - col0);
    if (rows <= 0) return;
    const int quads = cols / 4;                      // N is a multiple of 16
    const int64_t MN = (int64_t)M * N;
    for (int i = threadIdx.x; i < rows * quads; i += 256) {
        const int r = i / quads, q = i - r * quads;
        const int64_t at = (int64_t)(row0 + r) * N + col0 + q * 4;
        f32x4 v = *reinterpret_cast<const f32x4*>(partial + at);
        for (int s = 1; s < tail_splits; ++s) {
            const f32x4 o = *reinterpret_cast<const f32x4*>(partial + (int64_t)s * MN + at);
            v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
        }
        *reinterpret_cast<u32x2*>(C + at) = pack4<ACT>(v);
    }
}

// bfloat16 rows -> binary16 rows divided by a power of two per row (see FQ_BF16_VIA_F16): block r
// rewrites row r.  e = (exponent of the row's largest element) - 14 (between -141 and 114: every bfloat16
// magnitude is brought to 2^14 .. 2^15, an exact scaling);
// A16[r, :] = A[r, :] * 2^-e rounded to binary16, rowscale[r] = e as a float (2^e itself need not be a
// normal binary32 number; the product kernel applies it in two halves).
template <int THREADS>   // (a template so that every translation unit may hold a copy)
__global__ __launch_bounds__(THREADS) void fq_rows_to_f16_kernel(const uint16_t* __restrict__ A, int K,
                                                             uint16_t* __restrict__ A16,
                                                             float* __restrict__ rowscale) {
    __shared__ uint32_t red[4];
    const int64_t r = blockIdx.x;
    const u32x4* src = reinterpret_cast<const u32x4*>(A + r * K);
    u32x4* dst = reinterpret_cast<u32x4*>(A16 + r * K);
    const int units = K / 8;
    uint32_t m = 0;
    static_assert(THREADS == 256, "four waves are reduced below");
    for (int u = threadIdx.x; u < units; u += 256) {
        const u32x4 v = src[u];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t a0 = v[i] & 0x7fffu, a1 = (v[i] >> 16) & 0x7fffu;
            m = a0 > m ? a0 : m;
            m = a1 > m ? a1 : m;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t t = (uint32_t)__shfl_xor((int)m, o, 64);
        m = t > m ? t : m;
    }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = red[0];
#pragma unroll
    for (int i = 1; i < 4; ++i) m = red[i] > m ? red[i] : m;
    const int e = (int)(m >> 7) - 127 - 14;
    if (threadIdx.x == 0) rowscale[r] = (float)e;
    for (int u = threadIdx.x; u < units; u += 256) {
        const u32x4 v = src[u];
        u32x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float f0 = ldexpf(bitcast<float>(v[i] << 16), -e);
            const float f1 = ldexpf(bitcast<float>(v[i] & 0xffff0000u), -e);
            const f16x2 h = {(_Float16)f0, (_Float16)f1};
            o[i] = bitcast<uint32_t>(h);
        }
        dst[u] = o;
    }
}

// Largest scale of a bfloat16 scale matrix (FQ_BF16S_VIA_F16), in two steps without atomics: every block
// writes the largest bit pattern it saw, then one block folds those and writes 2^-E and 2^E (E = exponent of
// the largest scale, kept within +-120; 0 for an all-zero matrix) to out2[0], out2[1].
template <int THREADS>
__global__ __launch_bounds__(THREADS) void fq_scale_max_kernel(const uint16_t* __restrict__ scales, int64_t count,
                                                               uint32_t* __restrict__ part) {
    static_assert(THREADS == 256, "four waves are reduced below");
    __shared__ uint32_t red[4];
    uint32_t m = 0;
    const int64_t units = count / 8;                               // the scale matrix is a multiple of 16 wide
    for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < units; u += (int64_t)gridDim.x * 256) {
        const u32x4 v = reinterpret_cast<const u32x4*>(scales)[u];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t a0 = v[i] & 0x7fffu, a1 = (v[i] >> 16) & 0x7fffu;
            m = a0 > m ? a0 : m;
            m = a1 > m ? a1 : m;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t t = (uint32_t)__shfl_xor((int)m, o, 64);
        m = t > m ? t : m;
    }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < 4; ++i) m = red[i] > m ? red[i] : m;
        part[blockIdx.x] = m;
    }
}
template <int THREADS>
__global__ __launch_bounds__(THREADS) void fq_scale_exp_kernel(const uint32_t* __restrict__ part, int nparts,
                                                               float* __restrict__ out2) {
    if (threadIdx.x != 0) return;
    uint32_t m = 0;
    for (int i = 0; i < nparts; ++i) m = part[i] > m ? part[i] : m;
    int e = m == 0 ? 0 : (int)(m >> 7) - 127;
    e = e < -120 ? -120 : (e > 120 ? 120 : e);
    out2[0] = ldexpf(1.0f, -e);
    out2[1] = ldexpf(1.0f, e);
}

// s_waitcnt vmcnt(N) only (the other counters left alone); gfx9 encoding: vmcnt in bits 3:0 and 15:14
template <int N>
__device__ inline void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// KREC = k-blocks of the packed layout that make one k-block of this kernel (lane records per column tile
// and k-block): 2 for 8-bit codes in the 128-row shape, whose 64-row layout blocks would otherwise pay the
// barrier, the waits and the address arithmetic of a k-block for half as many MFMAs.
template <int ACT, int BITS, int MT, int NT, int WAVES, int SR, bool GROUPED, int PIPE, bool POST = false,
          int KREC = 1>
__global__ __launch_bounds__(WAVES * 64, (POST && MT == 2 && WAVES == 4 && ACT == FQ_F16) ? 3 : 1) void fq_gemm_mma_kernel(
    const uint16_t* __restrict__ A, const u32x4* __restrict__ codes, const uint16_t* __restrict__ scales,
    uint16_t* __restrict__ C, float* __restrict__ partial, int M, int N, int K, int g, int kb_per_split,
    int splits, int nblocks_n, int nblocks_m, int64_t codes_stride16, int64_t scales_stride,
    fq_group_items items, int tail_tiles, int tail_splits, int tail_kbs, const float* __restrict__ rowscale) {
    constexpr int KBLK = fq_kblk(BITS) * KREC;
    constexpr int STEPS = KBLK / FQ_KSTEP;
    constexpr int SPR = STEPS / KREC;            // k-steps per lane record
    constexpr int KC = KBLK / 8;
    constexpr int BM = MT * 16;
    constexpr int UNITS = BM * KC;
    static_assert(KREC == 1 || (PIPE > 0 && !POST), "several records per k-block: pipelined, pre-scaled form only");
    // LDS layout of the activation tile in the two-buffer form (the pipelined form has its own, below),
    // in 16-byte units: unit(kc, row) = kc * BM + (row ^ swz(kc)),
    // swz(kc) = kc * (16 / KC) mod 16.  A fragment read (16 rows of one kc per 16 lanes) then covers
    // one aligned 256-byte span, and a staging write (the KC units of a row in neighbouring lanes)
    // spreads over all banks; a padded pitch keeps the writes conflict-free but halves the read rate.
    constexpr int SWZ = 16 / KC;
    constexpr int NTHR = WAVES * 64;
    constexpr int UPT = (UNITS + NTHR - 1) / NTHR;
    // SR = scale rows a k-block spans: 1 when the group size is a multiple of KBLK, else KBLK / g
    // (or one per 32-row k-step when g does not divide KBLK)
    constexpr int SROWS = SR;
    static_assert(SR >= 1 && SR <= STEPS && STEPS % SR == 0, "");
    extern __shared__ u32x4 lds[];   // [PIPE ? PIPE + 1 : 2][KC * BM]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ntiles = N / FQ_NTILE;
    const int KB = K / KBLK;
    const int ml = lane & 15, j = lane >> 4;
    const int64_t kb_stride = (int64_t)ntiles * 64;

    // Block -> (n-block, m-block).  Consecutive block ids are dealt round-robin to the 8 XCDs,
    // each with its own L2; the ids an XCD receives are mapped to one contiguous run of logical
    // tiles, and logical tiles walk panels of PW n-blocks x all m-blocks, so that the blocks
    // resident on an XCD at one time share activation rows and weight columns in its L2.
    // With tail_tiles > 0 (and splits == 1) the first tiles run over all of K and write C; each of
    // the last tail_tiles tiles is shared by tail_splits blocks that write binary32 partial tiles
    // (they take the place of the partly filled last round of blocks).
    int bn, bm_idx, split, kb0, kb1;
    bool partial_out;
    {
        const int tiles = nblocks_n * nblocks_m;
        int bid = blockIdx.x;
        int L;
        auto spread = [](int b, int count) {   // ids an XCD receives -> one contiguous run of logical tiles
            return (count & 7) == 0 ? (b & 7) * (count >> 3) + (b >> 3) : b;
        };
        const int head = tiles - tail_tiles;
        if (tail_tiles == 0) {
            split = bid / tiles;
            bid -= split * tiles;
            L = spread(bid, tiles);
            kb0 = split * kb_per_split;
            kb1 = min(KB, kb0 + kb_per_split);
            partial_out = splits > 1;
        } else if (bid < head) {
            split = 0;
            L = spread(bid, head);
            kb0 = 0;
            kb1 = KB;
            partial_out = false;
        } else {
            const int r = bid - head;
            L = head + r / tail_splits;
            split = r - (r / tail_splits) * tail_splits;
            kb0 = split * tail_kbs;
            kb1 = min(KB, kb0 + tail_kbs);
            partial_out = true;
        }
        fq_tile_of(L, nblocks_n, nblocks_m, bn, bm_idx);
    }

    int64_t row0;
    int rows;
    if constexpr (GROUPED) {
        row0 = items.row0[bm_idx];
        rows = items.rows[bm_idx];
        const int e = items.expert[bm_idx];
        codes += (int64_t)e * codes_stride16;
        scales += (int64_t)e * scales_stride;
    } else {
        row0 = (int64_t)bm_idx * BM;
        rows = (int)min((int64_t)BM, (int64_t)M - row0);
    }

    constexpr int RB = fq_rec_bytes(BITS);
    const char* wbase[NT];
    const uint16_t* sbase[NT];
    bool tvalid[NT];
    const int tile0 = (bn * WAVES + wave) * NT;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tile = tile0 + nt;
        tvalid[nt] = tile < ntiles;
        const int tc = tvalid[nt] ? tile : 0;
        wbase[nt] = reinterpret_cast<const char*>(codes) + fq_rec(tc, 0, ntiles, 0) * RB;
        sbase[nt] = scales + tc * FQ_NTILE;
    }

    // activation staging: unit u = tid + NTHR r  ->  (row = u / KC, kc = u % KC)
    uint32_t a_off[UPT];     // element offset of the unit inside A (relative to row0, k = 0)
    int a_dst[UPT];
    bool a_ok[UPT];
#pragma unroll
    for (int r = 0; r < UPT; ++r) {
        const int u = tid + NTHR * r;
        const int row = u / KC, kc = u % KC;
        a_ok[r] = (u < UNITS) && (row < rows);
        a_off[r] = (uint32_t)(a_ok[r] ? row : 0) * (uint32_t)K + (uint32_t)kc * 8u;
        a_dst[r] = (u < UNITS) ? kc * BM + (row ^ ((kc * SWZ) & 15)) : -1;
    }
    const uint16_t* Arow = A + row0 * K;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint32_t magic = Dequant<ACT, BITS>::init();
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    // FQ_BF16S_VIA_F16: the two floats behind the M row scales are 2^-E and 2^E (E: exponent of the largest scale)
    float sshift = 1.0f;
    int sback_exp = 0;       // E
    if constexpr (ACT == FQ_BF16S_VIA_F16) {
        sshift = rowscale[M];
        sback_exp = (int)((bitcast<uint32_t>(rowscale[M + 1]) >> 23) & 255u) - 127;   // 2^E is a normal number
    }
    constexpr int NQ = KREC * NT;                // lane records of a k-block: [record][column tile]
    u32x4 wq[NQ], wq_n[NQ], areg[UPT];
    // Scale registers: one per (scale row, column tile), or, with four scale rows per k-block,
    // two rows per register (low / high half, filled by 16-bit loads into register halves).
    // POST (few rows per block, where the conversion and not the matrix pipe sets the pace): the codes
    // are converted without their scale (half the vector instructions for bf16), each scale group
    // is accumulated apart and folded into the result as acc += s * (p - OFFSET * rowsum), the row
    // sums of the activations coming from one more MFMA against an all-ones operand.  A lane then
    // needs the scales of its four output columns 4j .. 4j+3: one 8-byte register pair per (scale
    // row, column tile).
    static_assert(!POST || PIPE > 0, "the post-scaled form exists in the pipelined kernel only");
    constexpr int SPK = (!POST && SROWS >= 4) ? 2 : 1;      // scale rows packed per register
    constexpr int SREG = SROWS / SPK;
    typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
    typedef typename std::conditional<POST, u32x2, uint32_t>::type SC;
    SC sc[SREG][NT], sc_n[SREG][NT];
    // addresses are formed as (wave-uniform 64-bit base) + (32-bit lane offset), which the loads take as
    // they are (scalar base + vector offset), instead of 64-bit vector arithmetic per load
    // (used by the 128-row shapes; in the lower ones it costs registers they do not have)
    constexpr bool SADDR = MT == 8;
    const uint32_t lane_rec = (uint32_t)lane * RB;
    auto load_q = [&](u32x4 (&q)[NQ], int kb) {
#pragma unroll
        for (int r = 0; r < KREC; ++r) {
            const int64_t lkb = (int64_t)kb * KREC + r;      // k-block of the packed layout
            if constexpr (SADDR) {
                const int64_t kb_bytes = lkb * kb_stride * RB;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    q[r * NT + nt] = load_rec<BITS, false>(scalar_ptr(wbase[nt] + kb_bytes) + lane_rec);
            } else {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    q[r * NT + nt] = load_rec<BITS, false>(wbase[nt] + (lkb * kb_stride + lane) * RB);
            }
        }
    };
    auto load_s = [&](SC (&s)[SREG][NT], int kb) {
#pragma unroll
        for (int r = 0; r < SREG; ++r) {
            if constexpr (POST) {
                const int64_t srow = (int64_t)((kb * KBLK + r * (KBLK / SROWS)) / g) * N;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    s[r][nt] = *reinterpret_cast<const u32x2*>(sbase[nt] + srow + 4 * j);
            } else if constexpr (SPK == 1) {
                const int64_t srow = (int64_t)((kb * KBLK + r * (KBLK / SROWS)) / g) * N;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) s[r][nt] = SADDR ? scalar_ptr(sbase[nt] + srow)[(uint32_t)ml] : sbase[nt][srow + ml];
            } else {
                const int64_t srow0 = (int64_t)((kb * KBLK + (2 * r) * (KBLK / SROWS)) / g) * N;
                const int64_t srow1 = (int64_t)((kb * KBLK + (2 * r + 1) * (KBLK / SROWS)) / g) * N;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    u16x2 pr;
                    pr[0] = SADDR ? scalar_ptr(sbase[nt] + srow0)[(uint32_t)ml] : sbase[nt][srow0 + ml];
                    pr[1] = SADDR ? scalar_ptr(sbase[nt] + srow1)[(uint32_t)ml] : sbase[nt][srow1 + ml];
                    s[r][nt] = bitcast<uint32_t>(pr);
                }
            }
        }
    };
    auto load_w = [&](u32x4 (&q)[NQ], SC (&s)[SREG][NT], int kb) {
        load_q(q, kb);
        load_s(s, kb);
    };
    auto load_a = [&](int kb) {
        const uint16_t* base = Arow + (int64_t)kb * KBLK;
#pragma unroll
        for (int r = 0; r < UPT; ++r) areg[r] = *reinterpret_cast<const u32x4*>(base + a_off[r]);
    };
    // Rows past the end of the matrix load row 0 (always valid) and are zeroed here: a load under
    // a condition would hide the number of loads in flight from the wait-count bookkeeping, and
    // every later wait would then drain all of them.
    auto store_a = [&](u32x4* dst) {
#pragma unroll
        for (int r = 0; r < UPT; ++r)
            if (a_dst[r] >= 0) dst[a_dst[r]] = a_ok[r] ? areg[r] : zero4;
    };
    uint32_t s2c[NT];   // widened scale of the scale row under way, per column tile
    auto convert = [&](const u32x4 (&q)[NQ], const SC (&s)[SREG][NT], int t, int nt) -> u32x4 {
        const u32x4& rec = q[(t / SPR) * NT + nt];   // the record that holds k-step t
        const int ts = t % SPR;                      // ... as its step ts
        if constexpr (POST) {
            if (ts == 0) return Dequant<ACT, BITS>::template run<0>(rec, magic);
            if (ts == 1) return Dequant<ACT, BITS>::template run<1>(rec, magic);
            if (SPR > 2 && ts == 2) return Dequant<ACT, BITS>::template run<2 % SPR>(rec, magic);
            return Dequant<ACT, BITS>::template run<3 % SPR>(rec, magic);
        } else {
            // The scale is widened once per scale row and column tile (the k-steps of a row come one
            // after the other, the first of them first) and kept in s2c.  Its stored form stays opaque
            // until then: otherwise the widening is moved to the end of the previous k-block, and with
            // it the wait for the scale's load.
            const int srow = t / (STEPS / SROWS);
            if (t % (STEPS / SROWS) == 0) {
                uint32_t h = s[srow / SPK][nt];
                asm volatile("" : "+v"(h));
                if (SPK == 2 && (srow & 1)) h >>= 16;
                s2c[nt] = scale_operand<ACT>((uint16_t)h, sshift);
            }
            const uint32_t s2 = s2c[nt];
            if (ts == 0) return DequantScaled<ACT, BITS>::template run<0>(rec, magic, s2);
            if (ts == 1) return DequantScaled<ACT, BITS>::template run<1>(rec, magic, s2);
            if (SPR > 2 && ts == 2) return DequantScaled<ACT, BITS>::template run<2 % SPR>(rec, magic, s2);
            return DequantScaled<ACT, BITS>::template run<3 % SPR>(rec, magic, s2);
        }
    };

    constexpr int NFR = STEPS * MT;
    constexpr int APD = NFR >= 8 ? 3 : 1;   // fragments read ahead of their MFMAs
    static_assert(NFR % (APD + 1) == 0, "the fragment window must wrap at a k-block boundary");
    static_assert(STEPS % 2 == 0, "fragment sets alternate per k-step");
    constexpr int abuf_units = KC * BM;
    int a_rd[STEPS];   // unit of this lane's fragment row for k-step t (row tile 0)
#pragma unroll
    for (int t = 0; t < STEPS; ++t) a_rd[t] = (4 * t + j) * BM + (ml ^ (((4 * t + j) * SWZ) & 15));
    u32x4 w[2][NT];
    u32x4 afr[APD + 1];

    if constexpr (PIPE > 0) {
        // PIPE = D >= 2: the k loop is one software pipeline, D k-blocks deep, that does not drain at
        // k-block boundaries.  Slot i = t * MT + mt of a k-block holds the NT MFMAs of (k-step t, row
        // tile mt); around them:
        //   * the activation fragment of slot i + APD is read from LDS (from the next k-block's tile
        //     in the last APD slots), so the LDS latency is covered by matrix work;
        //   * the weights of k-step t + 1 are converted, one column tile per slot, into the other
        //     fragment set; in the last k-step these are the weights of step 0 of the next k-block;
        //   * D weight register sets: the set of k-block kb is reloaded with k-block kb + D as soon
        //     as its last conversion is done (slot W_SLOT); the sets take turns by unrolling the loop
        //     D times, so nothing in flight is ever copied;
        //   * D + 1 LDS tiles, filled straight from global memory (no registers, no staging stores):
        //     at BAR_SLOT the wave waits for its own share of tile kb + 1, the one barrier per
        //     k-block makes that tile visible, and the loads of tile kb + D are issued into the tile
        //     read during kb - 1, which every wave has finished before it arrives at that barrier.
        // LDS tile layout, in 16-byte units: unit(row, kc) = row * KC + (kc ^ swz(row)).  A wave-level
        // direct load fills 64 consecutive units = whole rows, each row a permutation of its own
        // contiguous 16 * KC bytes in global memory; a fragment read (16 rows of one kc) touches 16
        // different bank groups.  Rows past the end of the matrix load the last valid row; their
        // results are never stored.
        constexpr int D = PIPE;
        constexpr int NI = UNITS / 64;                  // wave-level direct loads per tile
        constexpr int DPT = NI >= WAVES ? NI / WAVES : 1;   // of which this wave issues DPT (or none)
        static_assert(UNITS % 64 == 0 && 64 % KC == 0 && (NI % WAVES == 0 || NI < WAVES),
                      "every wave issues the same number of direct loads, or none");
        static_assert(D >= 2, "");
        constexpr int BAR_SLOT = NFR - APD - 1;
        constexpr int W_SLOT = (STEPS - 2) * MT + (NT < MT ? NT : MT);   // after the last conversion from the set
        constexpr bool W_FIRST = W_SLOT <= BAR_SLOT;    // order of the two issue points inside a k-block
        constexpr int NWLOADS = NQ + SREG * SPK * NT;   // vector loads of one load_w
        // loads issued after those of tile kb + 1 and before the barrier of k-block kb
        constexpr int NYOUNGER = (D - 1) * NWLOADS + (D - 2) * DPT;
        static_assert(NYOUNGER < 64 && (D - 1) * (NWLOADS + DPT) < 64, "wait counter range");
        auto swz = [](int row) { return KC == 16 ? (row & 15) : ((row >> 1) & 7); };
        const bool a_loader = NI >= WAVES || wave < NI;   // wave-uniform
        uint32_t d_off[DPT];   // element offset inside A (relative to row0, k-block 0) of this lane's unit
#pragma unroll
        for (int r = 0; r < DPT; ++r) {
            const int u = (wave * DPT + r) * 64 + lane;
            const int row = u / KC, kcp = u % KC;
            const int rowc = row < rows ? row : rows - 1;
            d_off[r] = (uint32_t)rowc * (uint32_t)K + (uint32_t)((kcp ^ swz(row)) * 8);
        }
        auto load_a_lds = [&](int kb, int bufi) {
            if (!a_loader) return;
            const uint16_t* base = Arow + (int64_t)kb * KBLK;
            // Written as assembly on purpose: issued through the compiler's builtin, these loads make
            // its wait-count pass drain the whole memory queue (vmcnt(0)) at every later wait, which
            // would undo the weight prefetch.  The compiler's own waits stay correct without knowing
            // about them (the counter retires in order, so a wait for an older load only gets
            // stricter); the waits for these loads themselves are written out below.
            const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
                (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(lds + bufi * abuf_units + wave * DPT * 64));
#pragma unroll
            for (int r = 0; r < DPT; ++r) {
                const uint16_t* src = base + d_off[r];
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                             :
                             : "s"(lds_base + r * 1024), "v"(src)
                             : "memory", "m0");
            }
        };
#pragma unroll
        for (int t = 0; t < STEPS; ++t) a_rd[t] = ml * KC + ((4 * t + j) ^ swz(ml));

        u32x4 wqs[D][NQ];
        SC scs[D][SREG][NT];
        // POST: partial sums of the scale group at hand and the activations' row sums over it
        f32x4 pg[POST ? MT : 1][POST ? NT : 1], rsum[POST ? MT : 1];
        const f32x4 fzero = {0.f, 0.f, 0.f, 0.f};
        constexpr int GSTEPS = STEPS / SROWS;           // k-steps per scale row
        int cur = 0;
        if (kb0 < kb1) {
            // same issue order as inside the loop, so that the wait counts below hold from the start
            // (POST: the codes are reloaded at W_SLOT, the scales after the last fold of the k-block)
#pragma unroll
            for (int u = 0; u < D; ++u) {
                const int kbu = kb0 + u < kb1 ? kb0 + u : kb1 - 1;
                if (W_FIRST) load_q(wqs[u], kbu);
                if (W_FIRST && !POST) load_s(scs[u], kbu);
                load_a_lds(kbu, u);
                if (!W_FIRST) load_q(wqs[u], kbu);
                if (!W_FIRST || POST) load_s(scs[u], kbu);
            }
            wait_vmcnt<(D - 1) * (NWLOADS + DPT)>();   // tile 0 and weight set 0 have landed
            __syncthreads();
#pragma unroll
            for (int i = 0; i < APD; ++i) afr[i] = lds[a_rd[i / MT] + (i % MT) * 16 * KC];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) w[0][nt] = convert(wqs[0], scs[0], 0, nt);
        }
        // one k-block; (qa, sa) hold its weights, (qb, sb) those of the next one
        auto fold = [&](const SC (&sa)[SREG][NT], int srow, int mt) {
            if constexpr (POST) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    flush<ACT, BITS>(acc[mt][nt], pg[mt][nt], scales4<ACT>(sa[srow][nt]), rsum[mt][0]);
            }
        };
        auto kblock = [&](int kb, u32x4 (&qa)[NQ], SC (&sa)[SREG][NT], u32x4 (&qb)[NQ],
                          SC (&sb)[SREG][NT]) {
            const int nxt = cur == D ? 0 : cur + 1;
            const int last = cur == 0 ? D : cur - 1;     // the tile read during kb - 1
            const u32x4* abuf = lds + cur * abuf_units;
            const u32x4* nbuf = lds + nxt * abuf_units;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int i = t * MT + mt;
                    if (i == W_SLOT) {
                        if constexpr (POST) load_q(qa, kb + D < kb1 ? kb + D : kb1 - 1);
                        else load_w(qa, sa, kb + D < kb1 ? kb + D : kb1 - 1);
                    }
                    if (i == BAR_SLOT) {
                        // this wave's share of tile kb + 1 has landed once at most the loads issued
                        // after it are still in flight
                        wait_vmcnt<NYOUNGER>();
                        __syncthreads();
                        load_a_lds(kb + D < kb1 ? kb + D : kb1 - 1, last);
                    }
                    const int ip = i + APD;
                    if (ip < NFR) {
                        afr[ip % (APD + 1)] = abuf[a_rd[ip / MT] + (ip % MT) * 16 * KC];
                    } else {
                        afr[ip % (APD + 1)] = nbuf[a_rd[(ip - NFR) / MT] + ((ip - NFR) % MT) * 16 * KC];
                    }
#pragma unroll
                    for (int nt = mt; nt < NT; nt += MT) {
                        if (t + 1 < STEPS) w[(t + 1) & 1][nt] = convert(qa, sa, t + 1, nt);
                        else w[0][nt] = convert(qb, sb, 0, nt);
                    }
                    // keep the read and the conversion above where they are: without this the scheduler
                    // sinks them next to their uses and every fragment is then waited for
                    __builtin_amdgcn_sched_barrier(0);
                    const u32x4 a = afr[i % (APD + 1)];
                    if constexpr (POST) {
                        const bool first = t % GSTEPS == 0;
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            pg[mt][nt] = mfma16x16x32<ACT>(w[t & 1][nt], a, first ? fzero : pg[mt][nt]);
                        if constexpr (Dequant<ACT, BITS>::OFFSET != 0.0f)
                            rsum[mt] = mfma16x16x32<ACT>(ones_operand<ACT>(), a, first ? fzero : rsum[mt]);
                        // the group that ended in the slot before this one is folded in now, behind this
                        // slot's MFMAs, so that the fold does not wait for the matrix pipe
                        if (i > 0) {
                            const int tp = (i - 1) / MT, mp = (i - 1) % MT;
                            if ((tp + 1) % GSTEPS == 0) fold(sa, tp / GSTEPS, mp);
                        }
                    } else {
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = mfma16x16x32<ACT>(w[t & 1][nt], a, acc[mt][nt]);
                    }
                }
            }
            if constexpr (POST) {
                fold(sa, SROWS - 1, MT - 1);
                load_s(sa, kb + D < kb1 ? kb + D : kb1 - 1);
            }
            cur = nxt;
        };
        int kb = kb0;
        for (; kb + D <= kb1; kb += D) {
#pragma unroll
            for (int u = 0; u < D; ++u) kblock(kb + u, wqs[u], scs[u], wqs[(u + 1) % D], scs[(u + 1) % D]);
        }
#pragma unroll
        for (int u = 0; u < D - 1; ++u) {
            if (kb < kb1) {
                kblock(kb, wqs[u], scs[u], wqs[u + 1], scs[u + 1]);
                ++kb;
            }
        }
        // the last (redundant) direct loads still target this block's LDS: let them land before
        // the block can end and its LDS be given to another block
        wait_vmcnt<0>();
    } else {
        // Two LDS buffers, one barrier at the top of every k-block: a smaller footprint in LDS and
        // registers, so that two blocks fit a compute unit, which pays for the block shapes that
        // rely on several resident blocks (few rows, or 4 waves) rather than on one long pipeline.
        if (kb0 < kb1) {
            load_w(wq, sc, kb0);
            load_a(kb0);
        }
        int buf = 0;
        for (int kb = kb0; kb < kb1; ++kb) {
            store_a(lds + buf * abuf_units);
            __syncthreads();
            const int kbn = kb + 1 < kb1 ? kb + 1 : kb;
            load_w(wq_n, sc_n, kbn);
            load_a(kbn);
            const u32x4* abuf = lds + buf * abuf_units;
#pragma unroll
            for (int i = 0; i < APD; ++i) afr[i] = abuf[a_rd[i / MT] + (i % MT) * 16];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) w[0][nt] = convert(wq, sc, 0, nt);
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int i = t * MT + mt;
                    if (i + APD < NFR) {
                        const int ip = i + APD;
                        afr[ip % (APD + 1)] = abuf[a_rd[ip / MT] + (ip % MT) * 16];
                    }
                    if (t + 1 < STEPS) {
#pragma unroll
                        for (int nt = mt; nt < NT; nt += MT) w[(t + 1) & 1][nt] = convert(wq, sc, t + 1, nt);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    const u32x4 a = afr[i % (APD + 1)];
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[mt][nt] = mfma16x16x32<ACT>(w[t & 1][nt], a, acc[mt][nt]);
                }
            }
#pragma unroll
            for (int nt = 0; nt < NQ; ++nt) wq[nt] = wq_n[nt];
#pragma unroll
            for (int r = 0; r < SREG; ++r)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) sc[r][nt] = sc_n[r][nt];
            buf ^= 1;
        }
    }

#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int row = mt * 16 + ml;
        if (row >= rows) continue;
        if constexpr (ACT == FQ_BF16_VIA_F16 || ACT == FQ_BF16S_VIA_F16) {
            // Back from the row's power of two and the scales' common one: the result times 2^T, T = e + E.
            // 2^T may lie outside the normal binary32 range while the scaled result does not, so it is
            // applied as two normal factors 2^(T/2) (the value after the first one lies between the sum and
            // the result, hence in range whenever both are; exact unless the result itself is subnormal).
            int T = (int)rowscale[row0 + row] + sback_exp;
            T = T < -252 ? -252 : (T > 252 ? 252 : T);
            const int h1 = T >> 1, h2 = T - h1;
            const float m1 = bitcast<float>((uint32_t)(h1 + 127) << 23);
            const float m2 = bitcast<float>((uint32_t)(h2 + 127) << 23);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (acc[mt][nt] * m1) * m2;
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (!tvalid[nt]) continue;
            const int64_t n = (int64_t)(tile0 + nt) * FQ_NTILE + j * 4;
            if (!partial_out) {
                *reinterpret_cast<u32x2*>(C + (row0 + row) * N + n) = pack4<ACT>(acc[mt][nt]);
            } else {
                *reinterpret_cast<f32x4*>(partial + ((int64_t)split * M + row0 + row) * N + n) = acc[mt][nt];
            }
        }
    }
}

}  // namespace fqk

#endif  // FQ_GEMM_KERNELS_H_
