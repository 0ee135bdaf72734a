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
#include <stdint.h>

#include "fq_internal.h"
#include "fq_layout.h"

namespace {

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

template <int ACT>
__device__ inline f32x4 mfma16x16x32(const u32x4& w, const u32x4& a, const f32x4& c) {
    if constexpr (ACT == FQ_F16) {
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
template <int ACT, int BITS>
struct Dequant;

template <>
struct Dequant<FQ_F16, 4> {
    static constexpr float OFFSET = 0.0f;
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec) {
        const uint32_t w = rec[T];
        const uint32_t MAGIC = 0x64006400u;
        const uint32_t w8 = w >> 8;
        const f16x2 lo0 = bitcast<f16x2>((w & 0x000f000fu) | MAGIC);
        const f16x2 hi0 = bitcast<f16x2>((w & 0x00f000f0u) | MAGIC);
        const f16x2 lo1 = bitcast<f16x2>((w8 & 0x000f000fu) | MAGIC);
        const f16x2 hi1 = bitcast<f16x2>((w8 & 0x00f000f0u) | MAGIC);
        const f16x2 sub = {(_Float16)1032.0f, (_Float16)1032.0f};
        const f16x2 sc = {(_Float16)0.0625f, (_Float16)0.0625f};
        const f16x2 off = {(_Float16)-72.0f, (_Float16)-72.0f};
        u32x4 r;
        r[0] = bitcast<uint32_t>(lo0 - sub);                                 // elements 0,1
        r[1] = bitcast<uint32_t>(__builtin_elementwise_fma(hi0, sc, off));   // elements 2,3
        r[2] = bitcast<uint32_t>(lo1 - sub);                                 // elements 4,5
        r[3] = bitcast<uint32_t>(__builtin_elementwise_fma(hi1, sc, off));   // elements 6,7
        return r;
    }
};

template <>
struct Dequant<FQ_F16, 8> {
    static constexpr float OFFSET = 0.0f;
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec) {
        const uint32_t w0 = rec[2 * T], w1 = rec[2 * T + 1];
        const uint32_t MAGIC = 0x64646464u;
        const f16x2 sub = {(_Float16)1152.0f, (_Float16)1152.0f};   // 1024 + 128
        u32x4 r;
        r[0] = bitcast<uint32_t>(bitcast<f16x2>(__builtin_amdgcn_perm(MAGIC, w0, 0x04010400u)) - sub);
        r[1] = bitcast<uint32_t>(bitcast<f16x2>(__builtin_amdgcn_perm(MAGIC, w0, 0x04030402u)) - sub);
        r[2] = bitcast<uint32_t>(bitcast<f16x2>(__builtin_amdgcn_perm(MAGIC, w1, 0x04010400u)) - sub);
        r[3] = bitcast<uint32_t>(bitcast<f16x2>(__builtin_amdgcn_perm(MAGIC, w1, 0x04030402u)) - sub);
        return r;
    }
};

template <>
struct Dequant<FQ_BF16, 4> {
    static constexpr float OFFSET = 136.0f;
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec) {
        const uint32_t w = rec[T];
        const uint32_t MAGIC = 0x43004300u;
        u32x4 r;
        r[0] = (w & 0x000f000fu) | MAGIC;
        r[1] = ((w >> 4) & 0x000f000fu) | MAGIC;
        r[2] = ((w >> 8) & 0x000f000fu) | MAGIC;
        r[3] = ((w >> 12) & 0x000f000fu) | MAGIC;
        return r;
    }
};

template <>
struct Dequant<FQ_BF16, 8> {
    static constexpr float OFFSET = 128.0f;
    static __device__ inline uint32_t pair(uint32_t w, int lo_byte) {
        const float f0 = (float)((w >> (8 * lo_byte)) & 0xffu);
        const float f1 = (float)((w >> (8 * lo_byte + 8)) & 0xffu);
        // upper halves of the two binary32 values (exact: at most 8 significant bits)
        return __builtin_amdgcn_perm(bitcast<uint32_t>(f1), bitcast<uint32_t>(f0), 0x07060302u);
    }
    template <int T>
    static __device__ inline u32x4 run(const u32x4& rec) {
        const uint32_t w0 = rec[2 * T], w1 = rec[2 * T + 1];
        u32x4 r;
        r[0] = pair(w0, 0);
        r[1] = pair(w0, 2);
        r[2] = pair(w1, 0);
        r[3] = pair(w1, 2);
        return r;
    }
};

template <int ACT>
__device__ inline u32x4 ones_operand() {
    const uint32_t one2 = ACT == FQ_F16 ? 0x3c003c00u : 0x3f803f80u;
    u32x4 r = {one2, one2, one2, one2};
    return r;
}

__device__ inline f32x4 scales4(const uint16_t* p) {
    // four consecutive binary16 scales -> binary32
    const u32x2 v = *reinterpret_cast<const u32x2*>(p);
    const f16x2 a = bitcast<f16x2>(v[0]);
    const f16x2 b = bitcast<f16x2>(v[1]);
    f32x4 r = {(float)a[0], (float)a[1], (float)b[0], (float)b[1]};
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
// One wavefront = one independent worker: NT column tiles (16 NT columns) x one K range.
// It streams its tiles' records (NT KiB per k-block), reads the activation slice straight
// from L2 (M x KBLK values, shared by every wave of the chip), and needs no LDS or barrier
// in the main loop.  The four waves of a block take four consecutive K ranges of the same
// columns and add their results through LDS, so split-K costs a quarter of the partial
// traffic; remaining splits go through a binary32 partial buffer and a reduce kernel.
// PER_STEP = the scale changes inside a k-block (group size not a multiple of KBLK).
// ==========================================================================================
template <int ACT, int BITS, int NT, bool PER_STEP>
__global__ __launch_bounds__(256) void fq_gemm_skinny_kernel(
    const uint16_t* __restrict__ A, const u32x4* __restrict__ codes, const uint16_t* __restrict__ scales,
    uint16_t* __restrict__ C, float* __restrict__ partial, int M, int N, int K, int g, int kb_per_wave,
    int grid_splits) {
    constexpr int KBLK = BITS == 4 ? 128 : 64;
    constexpr int STEPS = KBLK / FQ_KSTEP;
    constexpr float OFF = Dequant<ACT, BITS>::OFFSET;
    __shared__ f32x4 red[3][NT][64];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int ntiles = N / FQ_NTILE;
    const int ngroups = (ntiles + NT - 1) / NT;
    const int ng = blockIdx.x % ngroups;
    const int gsplit = blockIdx.x / ngroups;          // < grid_splits
    const int KB = K / KBLK;
    const int kb0 = (gsplit * 4 + wave) * kb_per_wave;
    const int kb1 = min(KB, kb0 + kb_per_wave);
    const int m = lane & 15, j = lane >> 4;
    const bool mvalid = m < M;

    const u32x4* wp[NT];
    const uint16_t* sp[NT];
    bool tvalid[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tile = ng * NT + nt;
        tvalid[nt] = tile < ntiles;
        const int tc = tvalid[nt] ? tile : ng * NT;
        wp[nt] = codes + ((int64_t)tc * KB) * 64 + lane;
        sp[nt] = scales + tc * FQ_NTILE + j * 4;
    }
    const uint16_t* ap = A + (int64_t)(mvalid ? m : 0) * K + j * 8;

    f32x4 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 wq[NT], af[STEPS];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    if (kb0 < kb1) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wq[nt] = wp[nt][(int64_t)kb0 * 64];
#pragma unroll
        for (int t = 0; t < STEPS; ++t)
            af[t] = mvalid ? *reinterpret_cast<const u32x4*>(ap + (int64_t)kb0 * KBLK + t * FQ_KSTEP) : zero4;
    }
    for (int kb = kb0; kb < kb1; ++kb) {
        // prefetch the next k-block
        u32x4 wq_n[NT], af_n[STEPS];
        const int kbn = kb + 1 < kb1 ? kb + 1 : kb;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wq_n[nt] = wp[nt][(int64_t)kbn * 64];
#pragma unroll
        for (int t = 0; t < STEPS; ++t)
            af_n[t] = mvalid ? *reinterpret_cast<const u32x4*>(ap + (int64_t)kbn * KBLK + t * FQ_KSTEP) : zero4;

        if constexpr (!PER_STEP) {
            const int64_t srow = (int64_t)((kb * KBLK) / g) * N;
            f32x4 s[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) s[nt] = scales4(sp[nt] + srow);
            f32x4 p[NT];
            f32x4 psa = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) p[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
                u32x4 a;
                if (t == 0) a = af[0];
                if (t == 1) a = af[1];
                if (STEPS > 2 && t == 2) a = af[2 % STEPS];
                if (STEPS > 2 && t == 3) a = af[3 % STEPS];
                if constexpr (OFF != 0.0f) psa = mfma16x16x32<ACT>(ones_operand<ACT>(), a, psa);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    u32x4 w;
                    if (t == 0) w = Dequant<ACT, BITS>::template run<0>(wq[nt]);
                    if (t == 1) w = Dequant<ACT, BITS>::template run<1>(wq[nt]);
                    if (STEPS > 2 && t == 2) w = Dequant<ACT, BITS>::template run<2 % STEPS>(wq[nt]);
                    if (STEPS > 2 && t == 3) w = Dequant<ACT, BITS>::template run<3 % STEPS>(wq[nt]);
                    p[nt] = mfma16x16x32<ACT>(w, a, p[nt]);
                }
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) flush<ACT, BITS>(acc[nt], p[nt], s[nt], psa[0]);
        } else {
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
                const int64_t srow = (int64_t)((kb * KBLK + t * FQ_KSTEP) / g) * N;
                u32x4 a;
                if (t == 0) a = af[0];
                if (t == 1) a = af[1];
                if (STEPS > 2 && t == 2) a = af[2 % STEPS];
                if (STEPS > 2 && t == 3) a = af[3 % STEPS];
                f32x4 psa = {0.f, 0.f, 0.f, 0.f};
                if constexpr (OFF != 0.0f) psa = mfma16x16x32<ACT>(ones_operand<ACT>(), a, psa);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const f32x4 s = scales4(sp[nt] + srow);
                    u32x4 w;
                    if (t == 0) w = Dequant<ACT, BITS>::template run<0>(wq[nt]);
                    if (t == 1) w = Dequant<ACT, BITS>::template run<1>(wq[nt]);
                    if (STEPS > 2 && t == 2) w = Dequant<ACT, BITS>::template run<2 % STEPS>(wq[nt]);
                    if (STEPS > 2 && t == 3) w = Dequant<ACT, BITS>::template run<3 % STEPS>(wq[nt]);
                    f32x4 p = {0.f, 0.f, 0.f, 0.f};
                    p = mfma16x16x32<ACT>(w, a, p);
                    flush<ACT, BITS>(acc[nt], p, s, psa[0]);
                }
            }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wq[nt] = wq_n[nt];
#pragma unroll
        for (int t = 0; t < STEPS; ++t) af[t] = af_n[t];
    }

    // combine the four K ranges of the block
    if (wave > 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) red[wave - 1][nt][lane] = acc[nt];
    }
    __syncthreads();
    if (wave != 0 || !mvalid) return;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        f32x4 v = acc[nt];
#pragma unroll
        for (int w = 0; w < 3; ++w) {
            const f32x4 o = red[w][nt][lane];
            v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
        }
        if (!tvalid[nt]) continue;
        const int64_t n = (int64_t)(ng * NT + nt) * FQ_NTILE + j * 4;
        if (grid_splits == 1) {
            *reinterpret_cast<u32x2*>(C + (int64_t)m * N + n) = pack4<ACT>(v);
        } else {
            *reinterpret_cast<f32x4*>(partial + ((int64_t)gsplit * M + m) * N + n) = v;
        }
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

// ==========================================================================================
// Tiled kernel (any M): the prefill / batched case (section 4.1: in compute-bound cases
// the integer->float conversion, not the matrix-core math, is the bottleneck -- so each
// weight record is converted exactly once per block and reused for all BM rows).
//
// Block = 4 waves.  All four share one activation tile (BM = 16 MT rows x KBLK) staged
// through LDS with double buffering; wave w owns column tiles [4 bx + w) NT ... and converts
// only its own weights, straight from its global-load registers.
// LDS layout: 16-byte units (8 consecutive k of one row) at unit[kc * (BM + 1) + row];
// a fragment read is 16 lanes x 16 contiguous bytes per lane group.
// ==========================================================================================
struct fq_group_items {
    int count;
    int32_t row0[256];
    int16_t rows[256];
    int16_t expert[256];
};

template <int ACT, int BITS, int MT, int NT, bool PER_STEP, bool GROUPED>
__global__ __launch_bounds__(256) void fq_gemm_tile_kernel(
    const uint16_t* __restrict__ A, const u32x4* __restrict__ codes, const uint16_t* __restrict__ scales,
    uint16_t* __restrict__ C, float* __restrict__ partial, int M, int N, int K, int g, int kb_per_split,
    int splits, int64_t codes_stride16, int64_t scales_stride, fq_group_items items) {
    constexpr int KBLK = BITS == 4 ? 128 : 64;
    constexpr int STEPS = KBLK / FQ_KSTEP;
    constexpr int KC = KBLK / 8;             // 16-byte units per row and k-block
    constexpr int BM = MT * 16;
    constexpr int LDROW = BM + 1;
    constexpr int UNITS = BM * KC;
    constexpr int UPT = (UNITS + 255) / 256;  // units per thread
    constexpr float OFF = Dequant<ACT, BITS>::OFFSET;
    __shared__ u32x4 lds[2][KC * LDROW];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int ntiles = N / FQ_NTILE;
    const int KB = K / KBLK;
    const int split = blockIdx.z;
    const int kb0 = split * kb_per_split;
    const int kb1 = min(KB, kb0 + kb_per_split);
    const int ml = lane & 15, j = lane >> 4;

    int64_t row0;      // first row of this block in A / C
    int rows;          // valid rows in this block
    if constexpr (GROUPED) {
        const int it = blockIdx.y;
        row0 = items.row0[it];
        rows = items.rows[it];
        const int e = items.expert[it];
        codes += (int64_t)e * codes_stride16;
        scales += (int64_t)e * scales_stride;
    } else {
        row0 = (int64_t)blockIdx.y * BM;
        rows = (int)min((int64_t)BM, (int64_t)M - row0);
    }

    const u32x4* wp[NT];
    const uint16_t* sp[NT];
    bool tvalid[NT];
    const int tile0 = (blockIdx.x * 4 + wave) * NT;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tile = tile0 + nt;
        tvalid[nt] = tile < ntiles;
        const int tc = tvalid[nt] ? tile : 0;
        wp[nt] = codes + ((int64_t)tc * KB) * 64 + lane;
        sp[nt] = scales + tc * FQ_NTILE + j * 4;
    }

    // activation staging: unit u = tid + 256 r  ->  (row = u / KC, kc = u % KC)
    const uint16_t* a_src[UPT];
    int a_dst[UPT];
    bool a_ok[UPT];
#pragma unroll
    for (int r = 0; r < UPT; ++r) {
        const int u = tid + 256 * r;
        const int row = u / KC, kc = u % KC;
        a_ok[r] = (u < UNITS) && (row < rows);
        a_src[r] = A + (row0 + (a_ok[r] ? row : 0)) * K + kc * 8;
        a_dst[r] = (u < UNITS) ? kc * LDROW + row : -1;
    }

    f32x4 acc[MT][NT], p[MT][NT], psa[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        psa[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            p[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }

    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    u32x4 wq[NT], areg[UPT];
    if (kb0 < kb1) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wq[nt] = wp[nt][(int64_t)kb0 * 64];
#pragma unroll
        for (int r = 0; r < UPT; ++r)
            areg[r] = a_ok[r] ? *reinterpret_cast<const u32x4*>(a_src[r] + (int64_t)kb0 * KBLK) : zero4;
    }
    int buf = 0;
    for (int kb = kb0; kb < kb1; ++kb) {
#pragma unroll
        for (int r = 0; r < UPT; ++r)
            if (a_dst[r] >= 0) lds[buf][a_dst[r]] = areg[r];
        __syncthreads();
        // prefetch the next k-block into registers
        u32x4 wq_n[NT];
        const int kbn = kb + 1 < kb1 ? kb + 1 : kb;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wq_n[nt] = wp[nt][(int64_t)kbn * 64];
#pragma unroll
        for (int r = 0; r < UPT; ++r)
            areg[r] = a_ok[r] ? *reinterpret_cast<const u32x4*>(a_src[r] + (int64_t)kbn * KBLK) : zero4;

#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            u32x4 w[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                if (t == 0) w[nt] = Dequant<ACT, BITS>::template run<0>(wq[nt]);
                if (t == 1) w[nt] = Dequant<ACT, BITS>::template run<1>(wq[nt]);
                if (STEPS > 2 && t == 2) w[nt] = Dequant<ACT, BITS>::template run<2 % STEPS>(wq[nt]);
                if (STEPS > 2 && t == 3) w[nt] = Dequant<ACT, BITS>::template run<3 % STEPS>(wq[nt]);
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const u32x4 a = lds[buf][(t * 4 + j) * LDROW + mt * 16 + ml];
                if constexpr (OFF != 0.0f) psa[mt] = mfma16x16x32<ACT>(ones_operand<ACT>(), a, psa[mt]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) p[mt][nt] = mfma16x16x32<ACT>(w[nt], a, p[mt][nt]);
            }
            bool do_flush;
            int64_t srow;
            if constexpr (PER_STEP) {
                do_flush = true;
                srow = (int64_t)((kb * KBLK + t * FQ_KSTEP) / g) * N;
            } else {
                const int kend = (kb + 1) * KBLK;
                do_flush = (t == STEPS - 1) && (OFF != 0.0f || kend % g == 0 || kb == kb1 - 1);
                srow = (int64_t)((kb * KBLK) / g) * N;
            }
            if (do_flush) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const f32x4 s = scales4(sp[nt] + srow);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        flush<ACT, BITS>(acc[mt][nt], p[mt][nt], s, psa[mt][0]);
                        p[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) psa[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wq[nt] = wq_n[nt];
        buf ^= 1;
    }

#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int row = mt * 16 + ml;
        if (row >= rows) continue;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (!tvalid[nt]) continue;
            const int64_t n = (int64_t)(tile0 + nt) * FQ_NTILE + j * 4;
            if (splits == 1) {
                *reinterpret_cast<u32x2*>(C + (row0 + row) * N + n) = pack4<ACT>(acc[mt][nt]);
            } else {
                *reinterpret_cast<f32x4*>(partial + ((int64_t)split * M + row0 + row) * N + n) = acc[mt][nt];
            }
        }
    }
}

// ------------------------------------------------------------------------------ dispatch
constexpr int SKINNY_NT = 4;
constexpr int TILE_NT = 4;

template <int ACT, int BITS>
int launch_typed(const void* A, int64_t M, int64_t N, int64_t K, const void* codes, const void* scales,
                 int g, void* C, void* workspace, const fq_gemm_plan& plan, hipStream_t stream) {
    const int kblk = fq_kblk(BITS);
    const bool per_step = (g % kblk) != 0;
    const int ntiles = (int)(N / FQ_NTILE);
    float* partial = (float*)workspace;
    if (plan.kind == 0) {
        const int ngroups = (ntiles + SKINNY_NT - 1) / SKINNY_NT;
        const int grid_splits = plan.splits;
        dim3 grid((unsigned)(ngroups * grid_splits));
        auto kern = per_step ? fq_gemm_skinny_kernel<ACT, BITS, SKINNY_NT, true>
                             : fq_gemm_skinny_kernel<ACT, BITS, SKINNY_NT, false>;
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, stream, (const uint16_t*)A, (const u32x4*)codes,
                           (const uint16_t*)scales, (uint16_t*)C, partial, (int)M, (int)N, (int)K, g,
                           plan.kb_per_split, grid_splits);
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
    fq_gemm_plan p;
    const int kblk = fq_kblk(bits);
    const int KB = (int)(K / kblk);
    const int ntiles = (int)(N / FQ_NTILE);
    const int target_waves = 256 * 8;
    if (M <= 16) {
        p.kind = 0;
        p.mt = 1;
        const int ngroups = (ntiles + SKINNY_NT - 1) / SKINNY_NT;
        int want = (target_waves + ngroups - 1) / ngroups;         // K ranges wanted in total
        want = ((want + 3) / 4) * 4;
        if (want < 4) want = 4;
        int kbw = (KB + want - 1) / want;
        if (kbw < 1) kbw = 1;
        const int ranges = (KB + kbw - 1) / kbw;
        p.kb_per_split = kbw;                                       // per wave
        p.splits = (ranges + 3) / 4;                                // per grid (4 waves each)
    } else {
        p.kind = 1;
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
