// The integer path: int8 activations x int4 weights with integer group scales on the integer matrix cores
// (the paper's closing section names it as future work: "Conclusions and Limitations", last paragraph; the
// reading is stated in fq.h next to fq_quantize_w4a8).
//
//   weights      s[i, n] = z[i, n] * t[n],  z an integer in 1..16 (one byte per group), t binary16 per column;
//                codes q = int(w / s) as in Appendix A, stored in the packed 4-bit layout of fq_layout.h
//   activations  Appendix A at 8 bits per row: alpha[m] binary32, a[m, k] in [-127, 127]
//   product      S = sum_k a * (q * z) in int32 (v_mfma_i32_16x16x64_i8), C = alpha[m] * t[n] * S
//
// Packed layout of the codes of this path (its own: fq_unpack_w4a8 reads it back).  Tiles of 16 columns x 128
// rows, k-block-major, 64 lane records of 16 bytes per tile exactly like the floating-point layout
// (lane = 16 j + n % 16), but a record is ordered for v_mfma_i32_16x16x64_i8: MFMA step T (rows
// 64 T .. 64 T + 63 of the k-block) takes from lane group j the 16 consecutive rows 64 T + 16 j + 0..15;
// dword 2 T + h of the record holds rows 64 T + 16 j + 8 h + e (e = 0..7), byte b carrying element b in its
// low and element b + 4 in its high nibble (stored value q + 8).  Masking the low / the high nibbles of a
// dword then yields the operand's bytes in row order, and the activations need no reordering: lane (m, j)
// supplies the 16 consecutive int8 of row m at k = 64 T + 16 j.
//
// The weights are brought to the activation's type before the multiply, as section 4.1 describes for the
// floating-point kernels; here that type is int8 and the conversion is q * z, formed four at a time: the stored
// nibbles u = q + 8 of a dword are spread over bytes, one packed 16-bit multiply-add gives u * z + (128 - 8 z)
// in every byte (between 16 and 240: no carries), and flipping the top bit of each byte leaves q * z in two's
// complement.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <math.h>
#include <stdint.h>

#include "fq_gemm_kernels.h"
#include "fq_internal.h"
#include "fq_layout.h"

using namespace fqk;

namespace {

constexpr int ZMAX = 16;           // largest group multiplier: 7 * 16 = 112 fits an int8
constexpr float WLEVELS = 15.0f;   // 2^4 - 1, Appendix A
constexpr float ALEVELS = 255.0f;  // 2^8 - 1
constexpr int W8_NT = 3;           // column tiles per wave
constexpr int W8_WAVES = 8;

__device__ inline float f16_bits_to_float(uint16_t b) { return __half2float(__ushort_as_half(b)); }

// ------------------------------------------------------------------------------------------------------
// Weight quantiser, three small kernels (offline path):
//   1. abs-max of every group, as binary16 bit patterns, parked in the not-yet-written code buffer;
//   2. per column: t = smallest binary16 with 16 * 15 * t >= 2 * (largest group abs-max), then for every
//      group the smallest z in 1..16 with 15 * z * t >= 2 * (its abs-max)  (all products exact in binary32);
//   3. codes q = clamp(round_half_even(w / (z t)), -7, 7), IEEE binary32 quotient, packed.
// ------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void w8_group_absmax_kernel(const uint16_t* __restrict__ W, int64_t N, int g,
                                                               uint16_t* __restrict__ amax) {
    // thread (x, y): column x of the block's 64 columns, rows y, y + 4, ... of group blockIdx.y
    __shared__ uint16_t red[4][64];
    const int x = threadIdx.x & 63, y = threadIdx.x >> 6;
    const int64_t n = (int64_t)blockIdx.x * 64 + x;
    const int64_t grp = blockIdx.y;
    uint16_t m = 0;
    if (n < N) {
        const uint16_t* base = W + grp * g * N + n;
        for (int r = y; r < g; r += 4) {
            const uint16_t v = base[(int64_t)r * N] & 0x7fffu;
            m = v > m ? v : m;
        }
    }
    red[y][x] = m;
    __syncthreads();
    if (y == 0 && n < N) {
        for (int i = 1; i < 4; ++i) m = red[i][x] > m ? red[i][x] : m;
        amax[grp * N + n] = m;
    }
}

__global__ __launch_bounds__(256) void w8_scales_kernel(const uint16_t* __restrict__ amax, int64_t N, int groups,
                                                         uint8_t* __restrict__ z, uint16_t* __restrict__ tstep) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    uint16_t mcol = 0;
    for (int i = 0; i < groups; ++i) {
        const uint16_t v = amax[(int64_t)i * N + n];
        mcol = v > mcol ? v : mcol;
    }
    const float L = WLEVELS * (float)ZMAX;                                  // 240
    const float two_m = 2.0f * f16_bits_to_float(mcol);
    uint16_t tb = __half_as_ushort(__float2half_rn(__fdiv_rn(two_m, L)));   // nearest, then up if too small
    if (__fmul_rn(L, f16_bits_to_float(tb)) < two_m) tb += 1;
    tstep[n] = tb;
    const float t = f16_bits_to_float(tb);
    for (int i = 0; i < groups; ++i) {
        const float two_mi = 2.0f * f16_bits_to_float(amax[(int64_t)i * N + n]);
        int zi = 1;
        while (zi < ZMAX && __fmul_rn(WLEVELS * (float)zi, t) < two_mi) ++zi;   // (15 z) * t: exact
        z[(int64_t)i * N + n] = (uint8_t)zi;
    }
}

// row of the k-block that element e of dword d of lane group j holds
__host__ __device__ inline int w8_row(int d, int j, int e) { return 64 * (d >> 1) + 16 * j + 8 * (d & 1) + e; }

// one thread per lane record (16 bytes: 32 codes of one column in one k-block)
__global__ __launch_bounds__(256) void w8_encode_kernel(const uint16_t* __restrict__ W, int64_t K, int64_t N,
                                                         int g, const uint8_t* __restrict__ z,
                                                         const uint16_t* __restrict__ tstep,
                                                         uint32_t* __restrict__ codes) {
    const int64_t rec = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t ntiles = N / FQ_NTILE;
    if (rec >= (K / 128) * ntiles * 64) return;
    const int lane = (int)(rec & 63);
    const int64_t tile = (rec >> 6) % ntiles, kb = (rec >> 6) / ntiles;
    const int64_t n = tile * FQ_NTILE + (lane & 15);
    const int j = lane >> 4;
    const float t = f16_bits_to_float(tstep[n]);
    uint32_t out[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const int64_t k0 = kb * 128 + w8_row(d, j, 0);
        const float s = (float)z[(k0 / g) * N + n] * t;                      // exact; 8 rows inside one group
        uint32_t w = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float x = f16_bits_to_float(W[(k0 + e) * N + n]);
            int q = 0;
            if (s != 0.0f) q = (int)fminf(fmaxf(rintf(__fdiv_rn(x, s)), -7.0f), 7.0f);
            w |= (uint32_t)(q + 8) << (8 * (e & 3) + 4 * (e >> 2));
        }
        out[d] = w;
    }
    *reinterpret_cast<uint4*>(codes + rec * 4) = make_uint4(out[0], out[1], out[2], out[3]);
}

// the logical codes q[K, N] (int8) of a packed buffer: one thread per lane record
__global__ __launch_bounds__(256) void w8_unpack_kernel(const uint32_t* __restrict__ codes, int64_t K, int64_t N,
                                                         int8_t* __restrict__ q) {
    const int64_t rec = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t ntiles = N / FQ_NTILE;
    if (rec >= (K / 128) * ntiles * 64) return;
    const int lane = (int)(rec & 63);
    const int64_t tile = (rec >> 6) % ntiles, kb = (rec >> 6) / ntiles;
    const int64_t n = tile * FQ_NTILE + (lane & 15);
    const int j = lane >> 4;
    const uint4 v = *reinterpret_cast<const uint4*>(codes + rec * 4);
    const uint32_t d4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int e = 0; e < 8; ++e)
            q[(kb * 128 + w8_row(d, j, e)) * N + n] = (int8_t)((int)((d4[d] >> (8 * (e & 3) + 4 * (e >> 2))) & 0xfu) - 8);
}

// ------------------------------------------------------------------------------------------------------
// Activation quantiser: block r handles row r.  alpha = smallest binary32 with 255 alpha >= 2 max|A[r, :]|
// (nearest quotient, then one step up if the exact sign of 127.5 alpha - max, taken from a fused
// multiply-add, is negative); a = clamp(round_half_even(A / alpha), -127, 127), IEEE binary32 quotient.
// ------------------------------------------------------------------------------------------------------
template <int ACT>
__device__ inline float act_to_float(uint16_t b) {
    if constexpr (ACT == FQ_F16) return f16_bits_to_float(b);
    else return __uint_as_float((uint32_t)b << 16);
}

template <int ACT>
__global__ __launch_bounds__(256) void w8_act_quant_kernel(const uint16_t* __restrict__ A, int64_t K,
                                                            int8_t* __restrict__ Aq, float* __restrict__ alpha) {
    __shared__ uint32_t red[4];
    const int64_t r = blockIdx.x;
    const uint16_t* src = A + r * K;
    // rows of whole 16-byte units at 16-byte aligned addresses are read eight values and written eight bytes per
    // lane (with one value per lane the kernel is bound by the number of its memory instructions)
    const bool wide = (K & 7) == 0 && ((uintptr_t)A & 15) == 0 && ((uintptr_t)Aq & 7) == 0;
    const int64_t units = wide ? K >> 3 : 0;
    uint32_t m = 0;
    for (int64_t u = threadIdx.x; u < units; u += 256) {
        const u32x4 v = reinterpret_cast<const u32x4*>(src)[u];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t a0 = v[i] & 0x7fffu, a1 = (v[i] >> 16) & 0x7fffu;   // magnitudes of one format order
            m = a0 > m ? a0 : m;                                                // like their bit patterns
            m = a1 > m ? a1 : m;
        }
    }
    for (int64_t k = units * 8 + threadIdx.x; k < K; k += 256) {
        const uint32_t v = src[k] & 0x7fffu;
        m = v > m ? v : m;
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
    // 2 max / 255 = max / 127.5 (the same real number; this form cannot overflow for bfloat16 inputs near 2^128)
    const float amax = act_to_float<ACT>((uint16_t)m);
    float al = __fdiv_rn(amax, 0.5f * ALEVELS);
    if (__builtin_fmaf(0.5f * ALEVELS, al, -amax) < 0.0f) al = __uint_as_float(__float_as_uint(al) + 1u);   // next value up
    if (threadIdx.x == 0) alpha[r] = al;
    int8_t* dst = Aq + r * K;
    auto code = [&](uint16_t bits) -> uint32_t {
        int q = 0;
        if (al != 0.0f) q = (int)fminf(fmaxf(rintf(__fdiv_rn(act_to_float<ACT>(bits), al)), -127.0f), 127.0f);
        return (uint32_t)q & 0xffu;
    };
    for (int64_t u = threadIdx.x; u < units; u += 256) {
        const u32x4 v = reinterpret_cast<const u32x4*>(src)[u];
        u32x2 o;
#pragma unroll
        for (int h = 0; h < 2; ++h)
            o[h] = code((uint16_t)v[2 * h]) | (code((uint16_t)(v[2 * h] >> 16)) << 8) |
                   (code((uint16_t)v[2 * h + 1]) << 16) | (code((uint16_t)(v[2 * h + 1] >> 16)) << 24);
        reinterpret_cast<u32x2*>(dst)[u] = o;
    }
    for (int64_t k = units * 8 + threadIdx.x; k < K; k += 256) dst[k] = (int8_t)code(src[k]);
}

// ------------------------------------------------------------------------------------------------------
// Product.  Same orientation as the floating-point kernels: 16 x 16 tiles of C^T, the weights the first
// MFMA operand (16 columns n), the activations the second (16 rows m); a lane's packed record is, after the
// conversion, its slice of the first operand, so weights never pass through LDS.
// Block = 8 waves x 3 column tiles (384 columns), BM = 16 MT rows, k-block = 128 rows = two MFMA steps.
// The k loop is one software pipeline, two k-blocks deep:
//   * activation tiles (BM rows x 128 int8, natural order) go global -> LDS directly (global_load_lds_dwordx4),
//     three LDS tiles; the eight 16-byte units of a row are XOR-swizzled with the row (through the global
//     address each lane reads), so a fragment read of 16 rows of one unit column spreads over all banks;
//   * two weight register sets: the set of k-block kb is reloaded with k-block kb + 2 right after its last
//     conversion; the loop is unrolled twice so that the sets keep their names;
//   * one barrier per k-block, at its end: before it the wave waits until at most the loads issued after
//     those of k-block kb + 1 are in flight (the counter retires in order and every loading wave issues the
//     same loads), after it the tile read during kb is free.  Issue order inside k-block kb:
//     fragments of step 1 | MFMAs of step 0 with the conversion of step 1 between them | first MFMAs of step 1 |
//     A(kb + 2) into the tile read during kb - 1, W(kb + 2) | MFMAs of step 1 with the conversion of step 0 of
//     k-block kb + 1 between them; before the last of them: wait, barrier, fragments of step 0 of kb + 1.
// ZR = multiplier rows per k-block a lane needs: 1 when the group size is a multiple of 128, else one per
// 64-row step (the lane's 16 rows of a step lie inside one 32-row block, hence inside one group).
// With splits > 1 every block writes its int32 sums to its split's slab of a partial buffer and a second
// kernel adds the slabs (integers: exact whatever the order) and scales the sum.
// ------------------------------------------------------------------------------------------------------
typedef int v4i __attribute__((ext_vector_type(4)));
typedef uint16_t u16x2v __attribute__((ext_vector_type(2)));

// four stored nibbles spread over the bytes of x (each 1..15) -> four int8 values (u - 8) * z
__device__ inline uint32_t w8_scale_bytes(uint32_t x, u16x2v zz, u16x2v cc) {
    const u16x2v r = bitcast<u16x2v>(x) * zz + cc;          // u z + (128 - 8 z) in every byte, no carries
    return bitcast<uint32_t>(r) ^ 0x80808080u;
}

template <int OUT>
__device__ inline void w8_store4(uint16_t* C, const v4i& s, float scale_m, const float (&tn)[4]) {
    f32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (float)s[i] * (scale_m * tn[i]);
    *reinterpret_cast<u32x2*>(C) = pack4<OUT>(v);
}

template <int MT, int ZR, int OUT>
__global__ __launch_bounds__(W8_WAVES * 64) void fq_gemm_w4a8_kernel(
    const int8_t* __restrict__ Aq, const float* __restrict__ alpha, const u32x4* __restrict__ codes,
    const uint8_t* __restrict__ z, const uint16_t* __restrict__ tstep, uint16_t* __restrict__ C,
    int32_t* __restrict__ partial, int M, int N, int K, int g, int kb_per_split, int splits, int nblocks_n,
    int nblocks_m) {
    constexpr int NT = W8_NT;
    constexpr int BM = MT * 16;
    constexpr int UNITS = BM * 8;                       // 16-byte units of an activation tile
    constexpr int NI = UNITS / 64;                      // wave-level direct loads per tile
    constexpr int DPT = NI >= W8_WAVES ? NI / W8_WAVES : 1;   // of which this wave issues DPT (or none)
    constexpr int NW = NT + ZR * NT;                    // vector loads of one weight set
    static_assert(NI % W8_WAVES == 0 || NI < W8_WAVES, "every loading wave issues the same number of loads");
    extern __shared__ u32x4 lds[];                       // [3][UNITS]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ntiles = N / FQ_NTILE;
    const int KB = K / 128;
    const int ml = lane & 15, j = lane >> 4;
    const int64_t kb_stride = (int64_t)ntiles * 64;

    const int tiles = nblocks_n * nblocks_m;
    int bid = blockIdx.x;
    const int split = bid / tiles;
    bid -= split * tiles;
    // the block ids an XCD receives (every eighth) -> one contiguous run of logical tiles
    const int L = (tiles & 7) == 0 ? (bid & 7) * (tiles >> 3) + (bid >> 3) : bid;
    int bn, bm_idx;
    fq_tile_of(L, nblocks_n, nblocks_m, bn, bm_idx);
    const int kb0 = split * kb_per_split;
    const int kb1 = min(KB, kb0 + kb_per_split);
    const int64_t row0 = (int64_t)bm_idx * BM;
    const int rows = (int)min((int64_t)BM, (int64_t)M - row0);

    // wave-uniform bases (scalar registers); the lane's part is a 32-bit offset added by the load itself
    const char* wbase[NT];
    const uint8_t* zbase[NT];
    bool tvalid[NT];
    const int tile0 = (bn * W8_WAVES + wave) * NT;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tile = tile0 + nt;
        tvalid[nt] = tile < ntiles;
        const int tc = tvalid[nt] ? tile : 0;
        wbase[nt] = reinterpret_cast<const char*>(codes + fq_rec(tc, 0, ntiles, 0));
        zbase[nt] = z + (int64_t)tc * FQ_NTILE;
    }
    const uint32_t lane_rec = (uint32_t)lane * 16u;

    // direct loads: LDS unit u = (wave DPT + r) 64 + lane of a tile = (row u / 8, position u % 8), which holds
    // the row's 16-byte unit (position ^ (row & 7)); rows past the end repeat the last one (never stored)
    const bool a_loader = NI >= W8_WAVES || wave < NI;   // wave-uniform
    int64_t d_off[DPT];
#pragma unroll
    for (int r = 0; r < DPT; ++r) {
        const int u = (wave * DPT + r) * 64 + lane;
        const int row = u >> 3, pos = u & 7;
        const int rowc = row < rows ? row : rows - 1;
        d_off[r] = (row0 + rowc) * (int64_t)K + 16 * (pos ^ (row & 7));
    }
    auto load_a_lds = [&](int kb, int tile_i) {
        if (!a_loader) return;
        const int8_t* base = Aq + (int64_t)kb * 128;
        // (assembly on purpose: issued through the compiler's builtin these loads make its wait-count pass drain
        // the whole memory queue at every later wait; the waits for them are written out below)
        const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
            (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(lds + tile_i * UNITS + wave * DPT * 64));
#pragma unroll
        for (int r = 0; r < DPT; ++r) {
            const int8_t* src = base + d_off[r];
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                         :
                         : "s"(lds_base + r * 1024), "v"(src)
                         : "memory", "m0");
        }
    };
    int a_rd[2];
#pragma unroll
    for (int T = 0; T < 2; ++T) a_rd[T] = ml * 8 + ((4 * T + j) ^ (ml & 7));

    v4i acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = v4i{0, 0, 0, 0};

    u32x4 wqs[2][NT];
    uint32_t zqs[2][ZR][NT];
    auto load_w = [&](u32x4 (&q)[NT], uint32_t (&zr)[ZR][NT], int kb) {
        const int64_t kb_bytes = (int64_t)kb * kb_stride * 16;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) q[nt] = load_rec<4, false>(scalar_ptr(wbase[nt] + kb_bytes) + lane_rec);
#pragma unroll
        for (int r = 0; r < ZR; ++r) {
            if constexpr (ZR == 1) {
                // the k-block lies inside one group
                const int64_t zrow = (int64_t)((kb * 128) / g) * N;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) zr[r][nt] = scalar_ptr(zbase[nt] + zrow)[(uint32_t)ml];
            } else {
                // the group of this lane's 16 rows of step r
                const int64_t zrow = (int64_t)((kb * 128 + 64 * r + 16 * j) / g) * N;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) zr[r][nt] = zbase[nt][zrow + ml];
            }
        }
    };
    // piece p (0 .. 2 NT - 1) of the conversion of step T: dword h = p % 2 of column tile p / 2 (the pieces of a
    // step are converted in this order; the first piece of a column tile prepares its multiplier)
    uint32_t zcur[NT], ccur[NT];
    auto conv_piece = [&](u32x4 (&wop)[NT], const u32x4 (&q)[NT], const uint32_t (&zr)[ZR][NT], int T, int p) {
        const int nt = p >> 1, h = p & 1;
        if (h == 0) {
            // (the loaded multiplier stays opaque to the optimiser until here: otherwise its narrowing to 16 bits
            // is moved up to the load, and with it a wait for loads that were only just issued)
            uint32_t zi = zr[ZR == 1 ? 0 : T][nt];
            asm volatile("" : "+v"(zi));
            zcur[nt] = zi;
            ccur[nt] = (uint32_t)(0x8080 - (int)zi * 0x0808);   // 128 - 8 z in both bytes (8 z <= 128: no borrow)
        }
        const u16x2v zz = {(uint16_t)zcur[nt], (uint16_t)zcur[nt]};
        const u16x2v cc = {(uint16_t)ccur[nt], (uint16_t)ccur[nt]};
        const uint32_t w = q[nt][2 * T + h];
        wop[nt][2 * h] = w8_scale_bytes(w & 0x0f0f0f0fu, zz, cc);            // rows 8 h + 0..3
        wop[nt][2 * h + 1] = w8_scale_bytes((w >> 4) & 0x0f0f0f0fu, zz, cc);   // rows 8 h + 4..7
    };
    constexpr int NP = 2 * NT;                     // conversion pieces per step
    // the barrier stands before this MFMA group of step 1: early in the 128-row shape, so that the reads of the next
    // k-block's first fragments, which follow it, have six MFMA groups to return in (measured 1 - 4 % faster
    // than ahead of the last two groups; the tile it waits for was requested a k-block earlier either way)
    // (with two multiplier rows per k-block the fragments held that much longer cost spilled registers)
    constexpr int BAR_MT = MT >= 8 ? (ZR == 1 ? 1 : MT - 2) : (MT >= 4 ? MT - 2 : MT - 1);
    u32x4 wopA[NT], wopB[NT], af0[MT], af1[MT];
    // One k-block.  (qa, za): its weights, (qb, zb): those of k-block kb + 1, tile `cur`: its activations.
    // On entry wopA holds the converted operands of its step 0 and af0 that step's fragments (requested);
    // on exit the same for k-block kb + 1.  The conversions run in pieces between the MFMA groups (three MFMAs
    // of one row tile), where they issue while the matrix pipe works; with all conversions in front of the
    // MFMAs the waves of a block, which the barrier keeps in step, convert at the same time and multiply at the
    // same time, and the two units overlap for only a twentieth of the time.
    auto kblock = [&](int kb, int cur, u32x4 (&qa)[NT], uint32_t (&za)[ZR][NT], u32x4 (&qb)[NT],
                      uint32_t (&zb)[ZR][NT]) {
        const int kb2 = kb + 2 < kb1 ? kb + 2 : kb1 - 1;
        const int nxt = cur == 2 ? 0 : cur + 1;
        const u32x4* abuf = lds + cur * UNITS;
        const u32x4* nbuf = lds + nxt * UNITS;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af1[mt] = abuf[a_rd[1] + mt * 128];
        __builtin_amdgcn_sched_barrier(0);
        // step 0: MFMAs with wopA, conversion of step 1 into wopB
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bitcast<v4i>(wopA[nt]), bitcast<v4i>(af0[mt]),
                                                                    acc[mt][nt], 0, 0, 0);
            if (mt < NP) conv_piece(wopB, qa, za, 1, mt);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int p = MT; p < NP; ++p) conv_piece(wopB, qa, za, 1, p);
        __builtin_amdgcn_sched_barrier(0);
        // step 1: MFMAs with wopB, conversion of the next k-block's step 0 into wopA
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (mt == BAR_MT) {
                // every fragment of this tile has been read (own LDS reads returned), and this wave's share of
                // tile kb + 1 has landed once at most the loads issued after it are in flight
                // (with a single MFMA group per step the loads of k-block kb + 2 are issued behind this point:
                // then only the weights of kb + 1 are younger than its tile)
                __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0) only
                wait_vmcnt<(BAR_MT == 0 ? NW : DPT + NW)>();
                __syncthreads();
#pragma unroll
                for (int m2 = 0; m2 < MT; ++m2) af0[m2] = nbuf[a_rd[0] + m2 * 128];
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bitcast<v4i>(wopB[nt]), bitcast<v4i>(af1[mt]),
                                                                    acc[mt][nt], 0, 0, 0);
            if (mt < NP) conv_piece(wopA, qb, zb, 0, mt);
            __builtin_amdgcn_sched_barrier(0);
            if (mt == 0) {
                // Every register of the next k-block's weights is named here, so that the compiler places all
                // its waits for them in front of the loads issued now (they landed long ago); a wait placed
                // later would, in the compiler's count, which does not know of the direct loads, reach into the
                // loads just issued.  Set a is free.
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    asm volatile("" : : "v"(qb[nt][0]), "v"(qb[nt][1]), "v"(qb[nt][2]), "v"(qb[nt][3]));
#pragma unroll
                    for (int r = 0; r < ZR; ++r) asm volatile("" : : "v"(zb[r][nt]));
                }
                load_a_lds(kb2, cur >= 1 ? cur - 1 : 2);      // the tile read during kb - 1  (= (cur + 2) % 3)
                load_w(qa, za, kb2);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int p = MT; p < NP; ++p) conv_piece(wopA, qb, zb, 0, p);
        __builtin_amdgcn_sched_barrier(0);
    };

    if (kb0 < kb1) {
        const int kbn = kb0 + 1 < kb1 ? kb0 + 1 : kb1 - 1;
        // same issue order as inside the loop: A(kb), W(kb), A(kb + 1), W(kb + 1)
        load_a_lds(kb0, 0);
        load_w(wqs[0], zqs[0], kb0);
        load_a_lds(kbn, 1);
        load_w(wqs[1], zqs[1], kbn);
        wait_vmcnt<DPT + NW>();
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af0[mt] = lds[a_rd[0] + mt * 128];
#pragma unroll
        for (int p = 0; p < NP; ++p) conv_piece(wopA, wqs[0], zqs[0], 0, p);
        int kb = kb0, cur = 0;
        for (; kb + 2 <= kb1; kb += 2) {
            kblock(kb, cur, wqs[0], zqs[0], wqs[1], zqs[1]);
            cur = cur == 2 ? 0 : cur + 1;
            kblock(kb + 1, cur, wqs[1], zqs[1], wqs[0], zqs[0]);
            cur = cur == 2 ? 0 : cur + 1;
        }
        if (kb < kb1) kblock(kb, cur, wqs[0], zqs[0], wqs[1], zqs[1]);
        // the last (redundant) direct loads still target this block's LDS
        wait_vmcnt<0>();
    }

    float tn[NT][4];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            tn[nt][i] = tvalid[nt] ? f16_bits_to_float(tstep[(int64_t)(tile0 + nt) * FQ_NTILE + j * 4 + i]) : 0.0f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int row = mt * 16 + ml;
        if (row >= rows) continue;
        const float am = alpha[row0 + row];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (!tvalid[nt]) continue;
            const int64_t at = (row0 + row) * (int64_t)N + (int64_t)(tile0 + nt) * FQ_NTILE + j * 4;
            if (splits == 1) {
                w8_store4<OUT>(C + at, acc[mt][nt], am, tn[nt]);
            } else {
                *reinterpret_cast<v4i*>(partial + (int64_t)split * M * N + at) = acc[mt][nt];
            }
        }
    }
}


// ------------------------------------------------------------------------------------------------------
// Small-M kernel of the integer path (M <= 16), bound by the HBM read of the weights like its floating-point
// counterpart (fq_gemm_skinny_kernel), whose structure it takes: one block per compute unit and all blocks
// resident at once; a block is GP column groups x KW k-workers (run-time values), wave (gi, kw) owns NT
// column tiles and, in iteration `it`, k-block (sb * KW + kw) of super-block sb; codes and multipliers stream
// through a DEPTH-deep register ring per wave and never touch LDS; the int8 activation slice of a super-block
// (M rows x KW k-blocks of 128 bytes) is fetched once per block, DEPTH iterations ahead, through the same ring
// into one of two LDS buffers; one barrier per iteration; the k-workers' int32 sums are added through LDS
// (integer sums: exact in any order) and scaled by alpha[m] * t[n], or written as int32 slabs when K is
// also split over the grid (w8_finalize_kernel adds and scales those).
// ------------------------------------------------------------------------------------------------------
constexpr int W8S_PITCH = 17;      // LDS row pitch of the activation buffer in 16-byte units (16 rows + 1 pad)
constexpr int W8S_KC = 8;          // 16-byte activation units per row and k-block

template <int NT, int ZR, int AU>
struct W8Stage {
    u32x4 wq[NT];
    uint32_t zq[ZR][NT];
    u32x4 areg[AU];
};

template <int NT, int DEPTH, int ZR, int MAXW, int AU, int OUT>
__global__ __launch_bounds__(MAXW * 64) void fq_w4a8_skinny_kernel(
    const int8_t* __restrict__ Aq, const float* __restrict__ alpha, const u32x4* __restrict__ codes,
    const uint8_t* __restrict__ z, const uint16_t* __restrict__ tstep, uint16_t* __restrict__ C,
    int32_t* __restrict__ partial, int M, int N, int K, uint32_t g32, uint32_t g32_recip, int gp, int kw_n,
    int grid_splits) {
    constexpr int KC = W8S_KC, PITCH = W8S_PITCH;
    typedef W8Stage<NT, ZR, AU> Stage;
    extern __shared__ u32x4 lds[];   // two activation buffers [kw_n * KC][PITCH]; later the reduction

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
    const int KB = K / 128;
    const int SB = (KB + kw_n - 1) / kw_n;            // super-blocks of kw_n k-blocks
    const int n_it = gsplit < SB ? (SB - gsplit + grid_splits - 1) / grid_splits : 0;   // block-uniform
    const int64_t kb_stride = (int64_t)ntiles * 64;   // records between consecutive k-blocks of a tile
    const int ml = lane & 15, j = lane >> 4;
    const int abuf_units = kw_n * KC * PITCH;

    const char* wbase[NT];
    const uint8_t* zbase[NT];
    bool tvalid[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tile = ng * NT + nt;
        tvalid[nt] = gvalid && tile < ntiles;
        const int tc = tvalid[nt] ? tile : 0;
        wbase[nt] = reinterpret_cast<const char*>(codes + fq_rec(tc, 0, ntiles, 0));
        zbase[nt] = z + (int64_t)tc * FQ_NTILE + ml;
    }

    // cooperative activation fetch: unit u = tid + r * nthreads covers row u / upr, unit column u % upr of the
    // super-block (upr = kw_n * KC units of 16 int8 per row)
    const int upr = kw_n * KC;
    int a_row[AU], a_col[AU];
#pragma unroll
    for (int r = 0; r < AU; ++r) {
        const int u = tid + r * nthreads;
        a_row[r] = u / upr;
        a_col[r] = u - a_row[r] * upr;
    }

    v4i acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = v4i{0, 0, 0, 0};
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    auto load_act = [&](u32x4 (&areg)[AU], int it) {
        const int64_t k0 = (int64_t)(gsplit + it * grid_splits) * kw_n * 128;
#pragma unroll
        for (int r = 0; r < AU; ++r) {
            int64_t k = k0 + a_col[r] * 16;
            k = k < K ? k : K - 16;                      // past the end (tail super-block): never multiplied
            areg[r] = a_row[r] < M ? *reinterpret_cast<const u32x4*>(Aq + (int64_t)a_row[r] * K + k) : zero4;
        }
    };
    auto store_act = [&](const u32x4 (&areg)[AU], int buf) {
#pragma unroll
        for (int r = 0; r < AU; ++r)
            if (a_row[r] < 16) lds[buf * abuf_units + a_col[r] * PITCH + a_row[r]] = areg[r];
    };
    // stage `it`: this wave's codes and multipliers for iteration it, and the lane's share of the activations of
    // iteration it + 1
    auto load_stage = [&](Stage& sl, int it) {
        int kb = (gsplit + it * grid_splits) * kw_n + kw;
        kb = kb < KB ? kb : KB - 1;                      // tail super-block: idle workers re-read the last block
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) sl.wq[nt] = load_rec<4, true>(wbase[nt] + ((int64_t)kb * kb_stride + lane) * 16);
#pragma unroll
        for (int r = 0; r < ZR; ++r) {
            // group of the 32-row step at hand (ZR == 1: the k-block lies inside one group; else the group of this
            // lane's 16 rows of MFMA step r): an exact division by g / 32 as a multiplication by its rounded-up
            // reciprocal (valid while step * (g / 32) < 2^32)
            const uint32_t step = (uint32_t)kb * 4u + (ZR == 1 ? 0u : 2u * r + (uint32_t)(j >> 1));
            const uint32_t grp = g32 == 1 ? step : __umulhi(step, g32_recip);
            const int64_t zrow = (int64_t)grp * N;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) sl.zq[r][nt] = zbase[nt][zrow];
        }
        load_act(sl.areg, it + 1);
    };
    // one iteration: publish the next activations, read this iteration's fragments, convert and multiply
    auto iterate = [&](const Stage& sl, int it) {
        store_act(sl.areg, (it + 1) & 1);
        const int kb = (gsplit + it * grid_splits) * kw_n + kw;
        u32x4 af[2];
        const u32x4* abuf = lds + (it & 1) * abuf_units + (kw * KC + j) * PITCH + ml;
#pragma unroll
        for (int T = 0; T < 2; ++T) af[T] = abuf[T * 4 * PITCH];
        if (gvalid && kb < KB) {
#pragma unroll
            for (int T = 0; T < 2; ++T) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const uint32_t zi = sl.zq[ZR == 1 ? 0 : T][nt];
                    const uint32_t ci = (uint32_t)(0x8080 - (int)zi * 0x0808);   // 128 - 8 z in both bytes
                    const u16x2v zz = {(uint16_t)zi, (uint16_t)zi};
                    const u16x2v cc = {(uint16_t)ci, (uint16_t)ci};
                    u32x4 wop;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t w = sl.wq[nt][2 * T + h];
                        wop[2 * h] = w8_scale_bytes(w & 0x0f0f0f0fu, zz, cc);
                        wop[2 * h + 1] = w8_scale_bytes((w >> 4) & 0x0f0f0f0fu, zz, cc);
                    }
                    acc[nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bitcast<v4i>(wop), bitcast<v4i>(af[T]), acc[nt], 0, 0, 0);
                }
            }
        }
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

    // the k-workers' sums of each column group, added by all threads of the block (one result quad each)
    auto store_quad = [&](const v4i& v, int group, int nt, int ln) {
        const int mq = ln & 15, jq = ln >> 4;
        const int tile = group * NT + nt;
        if (mq >= M || group >= ngroups || tile >= ntiles) return;
        const int64_t n = (int64_t)tile * FQ_NTILE + jq * 4;
        if (grid_splits == 1) {
            float tn[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) tn[i] = f16_bits_to_float(tstep[n + i]);
            w8_store4<OUT>(C + (int64_t)mq * N + n, v, alpha[mq], tn);
        } else {
            *reinterpret_cast<v4i*>(partial + ((int64_t)gsplit * M + mq) * N + n) = v;
        }
    };
    if (kw_n == 1) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) store_quad(acc[nt], ng, nt, lane);
        return;
    }
    v4i* red = reinterpret_cast<v4i*>(lds);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) red[(wave * NT + nt) * 64 + lane] = acc[nt];
    __syncthreads();
    const int nquads = gp * NT * 64;
    for (int q = tid; q < nquads; q += nthreads) {
        const int gq = q / (NT * 64);            // column group of the block
        const int r = q - gq * (NT * 64);        // nt * 64 + lane inside the group
        const v4i* src = red + (int64_t)gq * kw_n * NT * 64 + r;   // worker w: + w * NT * 64
        v4i v = src[0];
#pragma unroll 4
        for (int w = 1; w < kw_n; ++w) v += src[w * NT * 64];
        store_quad(v, bx * gp + gq, r >> 6, r & 63);
    }
}

template <int OUT>
__global__ __launch_bounds__(256) void w8_finalize_kernel(const int32_t* __restrict__ S, int splits,
                                                           const float* __restrict__ alpha,
                                                           const uint16_t* __restrict__ tstep, int64_t M, int64_t N,
                                                           uint16_t* __restrict__ C) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= M * N) return;
    const int64_t m = i / N, n = i - m * N;                  // N is a multiple of 16: the four share a row
    v4i s = *reinterpret_cast<const v4i*>(S + i);
    for (int k = 1; k < splits; ++k) s += *reinterpret_cast<const v4i*>(S + (int64_t)k * M * N + i);
    float tn[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) tn[k] = f16_bits_to_float(tstep[n + k]);
    w8_store4<OUT>(C + i, s, alpha[m], tn);
}

struct w8_plan {
    int mt, splits, kb_per_split, nblocks_n, nblocks_m;
    int small, gp, kw, au;      // small-M kernel (M <= 16): column groups x k-workers per block, activation units per lane
};

constexpr int W8S_NT = 3, W8S_MAXW = 12;   // the small-M kernel that is compiled in
// ring depth: three stages where the registers allow it without spills (one multiplier row per k-block and one
// activation unit per lane: 164 registers; measured 4 - 6 % faster than two on the OPT-175B shapes), else two
constexpr int w8s_depth(int zr, int au) { return zr == 1 && au == 1 ? 3 : 2; }

w8_plan w8_plan_of(int64_t M, int64_t N, int64_t K) {
    w8_plan p = {};
    if (M <= 16) {
        // One block per compute unit, all resident at once; the block shape that fills the compute units most
        // evenly, scored like the floating-point small-M plan (evenness of the fill squared, bytes in flight per
        // compute unit up to 64 KiB, a second round of blocks, a split of K over the grid and lone k-workers cost).
        const int ncu = fq_cu_count();
        const int ntiles = (int)(N / FQ_NTILE);
        const int KB = (int)(K / 128);
        const int ngroups = (ntiles + W8S_NT - 1) / W8S_NT;
        p.small = 1;
        p.mt = 1;
        double best = -1.0;
        for (int gp = 1; gp <= W8S_MAXW; ++gp) {
            int kw = W8S_MAXW / gp;
            if (kw > KB) kw = KB;
            const int need = (int)M * W8S_KC;
            const int au = need <= 64 * gp ? 1 : (need <= 128 * gp ? 2 : 0);
            if (au == 0 || kw < 1) continue;
            const int64_t blocks = (ngroups + gp - 1) / gp;
            const int SB = (KB + kw - 1) / kw;
            int gs = 1;
            if (blocks <= ncu / 2) gs = (int)(ncu / blocks);
            if (gs > 8) gs = 8;
            if (gs > SB) gs = SB;
            const int64_t grid = blocks * gs;
            const int64_t rounds = (grid + ncu - 1) / ncu;
            const double eff = (double)ngroups * gs / (double)(rounds * ncu * gp);
            const double inflight = (double)(gp * kw) * W8S_NT * 2;   // KiB (with the shallower ring)
            double score = eff * eff * (inflight >= 64.0 ? 1.0 : sqrt(inflight / 64.0));
            score /= 1.0 + 0.1 * (double)(rounds - 1);
            if (au == 2) score *= 0.8;
            if (gs > 1) score *= 0.8;
            if (gp * kw < 6) score *= 0.85;
            if (kw == 1) score *= 0.95;
            if (score > best + 1e-9) {
                best = score;
                p.gp = gp;
                p.kw = kw;
                p.au = au;
                p.splits = gs;
            }
        }
        p.kb_per_split = 0;
        p.nblocks_n = (ngroups + p.gp - 1) / p.gp;
        p.nblocks_m = 1;
        return p;
    }
    p.mt = M <= 32 ? 2 : (M <= 64 ? 4 : 8);
    const int ntiles = (int)(N / FQ_NTILE);
    p.nblocks_n = (ntiles + W8_WAVES * W8_NT - 1) / (W8_WAVES * W8_NT);
    p.nblocks_m = (int)((M + p.mt * 16 - 1) / (p.mt * 16));
    const int64_t tiles = (int64_t)p.nblocks_n * p.nblocks_m;
    const int KB = (int)(K / 128);
    int splits = 1;
    if (tiles < 192) splits = (int)(256 / tiles);      // fill the compute units when there are few tiles
    if (splits > 8) splits = 8;
    if (splits > KB) splits = KB;
    p.kb_per_split = (KB + splits - 1) / splits;
    p.splits = (KB + p.kb_per_split - 1) / p.kb_per_split;
    return p;
}

int w8_check(int64_t K, int64_t N, int group_size, int* g_eff) {
    if (K <= 0 || N <= 0 || group_size < 0) return FQ_ERR_INVALID_ARG;
    const int64_t g = group_size == 0 ? K : (int64_t)group_size;
    if (g > K || K % g != 0) return FQ_ERR_INVALID_ARG;
    // K <= 131072 keeps every sum inside an int32: K * 127 * 112 < 2^31
    if (K > 131072 || N > (int64_t)1 << 24 || N % FQ_NTILE != 0 || K % 128 != 0 || g % 32 != 0) return FQ_ERR_UNSUPPORTED;
    *g_eff = (int)g;
    return FQ_OK;
}

template <int MT, int OUT>
void w8_launch(const w8_plan& p, int g, const int8_t* Aq, const float* alpha, const void* codes, const uint8_t* z,
               const void* tstep, void* C, int32_t* partial, int64_t M, int64_t N, int64_t K, hipStream_t stream) {
    const dim3 grid((unsigned)((int64_t)p.nblocks_n * p.nblocks_m * p.splits));
    const size_t lds = (size_t)3 * MT * 16 * 8 * 16;
    const int zr = g % 128 == 0 ? 1 : 2;
#define W8_GO(ZR_)                                                                                              \
    hipLaunchKernelGGL((fq_gemm_w4a8_kernel<MT, ZR_, OUT>), grid, dim3(W8_WAVES * 64), lds, stream, Aq, alpha,   \
                       (const u32x4*)codes, z, (const uint16_t*)tstep, (uint16_t*)C, partial, (int)M, (int)N,    \
                       (int)K, g, p.kb_per_split, p.splits, p.nblocks_n, p.nblocks_m)
    if (zr == 1) W8_GO(1);
    else W8_GO(2);
#undef W8_GO
}

template <int OUT, int ZR, int AU>
int w8_launch_small(const w8_plan& p, int g, const int8_t* Aq, const float* alpha, const void* codes, const uint8_t* z,
                    const void* tstep, void* C, int32_t* partial, int64_t M, int64_t N, int64_t K, hipStream_t stream) {
    const size_t lds_act = (size_t)2 * p.kw * W8S_KC * W8S_PITCH * 16;
    const size_t lds_red = (size_t)p.gp * p.kw * W8S_NT * 64 * 16;
    const size_t lds = lds_act > lds_red ? lds_act : lds_red;       // at most 36 KiB
    const uint32_t g32 = (uint32_t)(g / 32);
    const uint32_t g32_recip = (uint32_t)((((uint64_t)1 << 32) + g32 - 1) / g32);   // unused when g32 == 1
    hipLaunchKernelGGL((fq_w4a8_skinny_kernel<W8S_NT, w8s_depth(ZR, AU), ZR, W8S_MAXW, AU, OUT>),
                       dim3((unsigned)(p.nblocks_n * p.splits)), dim3((unsigned)(p.gp * p.kw * 64)), lds, stream, Aq,
                       alpha, (const u32x4*)codes, z, (const uint16_t*)tstep, (uint16_t*)C, partial, (int)M, (int)N,
                       (int)K, g32, g32_recip, p.gp, p.kw, p.splits);
    return FQ_OK;
}

template <int OUT>
int w8_gemm(const int8_t* Aq, const float* alpha, int64_t M, int64_t N, int64_t K, const void* codes, const uint8_t* z,
            const void* tstep, int g, void* C, void* workspace, hipStream_t stream) {
    const w8_plan p = w8_plan_of(M, N, K);
    int32_t* partial = (int32_t*)workspace;
    if (p.small) {
        const bool zr1 = g % 128 == 0;
        if (zr1 && p.au == 1) w8_launch_small<OUT, 1, 1>(p, g, Aq, alpha, codes, z, tstep, C, partial, M, N, K, stream);
        else if (zr1) w8_launch_small<OUT, 1, 2>(p, g, Aq, alpha, codes, z, tstep, C, partial, M, N, K, stream);
        else if (p.au == 1) w8_launch_small<OUT, 2, 1>(p, g, Aq, alpha, codes, z, tstep, C, partial, M, N, K, stream);
        else w8_launch_small<OUT, 2, 2>(p, g, Aq, alpha, codes, z, tstep, C, partial, M, N, K, stream);
    } else
    switch (p.mt) {
        case 2: w8_launch<2, OUT>(p, g, Aq, alpha, codes, z, tstep, C, partial, M, N, K, stream); break;
        case 4: w8_launch<4, OUT>(p, g, Aq, alpha, codes, z, tstep, C, partial, M, N, K, stream); break;
        default: w8_launch<8, OUT>(p, g, Aq, alpha, codes, z, tstep, C, partial, M, N, K, stream); break;
    }
    if (p.splits > 1) {
        const int64_t n4 = M * N / 4;
        hipLaunchKernelGGL(w8_finalize_kernel<OUT>, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, stream,
                           (const int32_t*)partial, p.splits, alpha, (const uint16_t*)tstep, M, N, (uint16_t*)C);
    }
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}

}  // namespace

extern "C" {

size_t fq_zscale_bytes(int64_t K, int64_t N, int group_size) {
    int g = 0;
    if (w8_check(K, N, group_size, &g) != FQ_OK) return 0;
    return (size_t)((K / g) * N);
}

int fq_quantize_w4a8(const void* W_f16, int64_t K, int64_t N, int group_size, void* codes, uint8_t* zscale,
                     void* tstep_f16, void* stream) {
    if (!W_f16 || !codes || !zscale || !tstep_f16) return FQ_ERR_INVALID_ARG;
    int g = 0;
    const int st = w8_check(K, N, group_size, &g);
    if (st != FQ_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int groups = (int)(K / g);
    if (groups > 65535) return FQ_ERR_UNSUPPORTED;
    uint16_t* amax = (uint16_t*)codes;      // K N / 2 bytes hold the K / g x N abs-max values (g >= 32)
    hipLaunchKernelGGL(w8_group_absmax_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)groups), dim3(256), 0, s,
                       (const uint16_t*)W_f16, N, g, amax);
    hipLaunchKernelGGL(w8_scales_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, (const uint16_t*)amax, N,
                       groups, zscale, (uint16_t*)tstep_f16);
    const int64_t recs = (K / 128) * (N / FQ_NTILE) * 64;
    hipLaunchKernelGGL(w8_encode_kernel, dim3((unsigned)((recs + 255) / 256)), dim3(256), 0, s, (const uint16_t*)W_f16, K,
                       N, g, (const uint8_t*)zscale, (const uint16_t*)tstep_f16, (uint32_t*)codes);
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}

int fq_unpack_w4a8(const void* codes, int64_t K, int64_t N, int8_t* q, void* stream) {
    if (!codes || !q) return FQ_ERR_INVALID_ARG;
    int g = 0;
    const int st = w8_check(K, N, 0, &g);
    if (st != FQ_OK) return st;
    const int64_t recs = (K / 128) * (N / FQ_NTILE) * 64;
    hipLaunchKernelGGL(w8_unpack_kernel, dim3((unsigned)((recs + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (const uint32_t*)codes, K, N, q);
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}

int fq_quantize_act_i8(const void* A, int act_dtype, int64_t M, int64_t K, int8_t* Aq, float* alpha, void* stream) {
    if (M < 0 || K <= 0) return FQ_ERR_INVALID_ARG;
    if (act_dtype != FQ_F16 && act_dtype != FQ_BF16) return FQ_ERR_INVALID_ARG;
    if (M == 0) return FQ_OK;
    if (!A || !Aq || !alpha) return FQ_ERR_INVALID_ARG;
    if (M > (int64_t)1 << 24 || K > (int64_t)1 << 24) return FQ_ERR_UNSUPPORTED;
    if (act_dtype == FQ_F16)
        hipLaunchKernelGGL(w8_act_quant_kernel<FQ_F16>, dim3((unsigned)M), dim3(256), 0, (hipStream_t)stream,
                           (const uint16_t*)A, K, Aq, alpha);
    else
        hipLaunchKernelGGL(w8_act_quant_kernel<FQ_BF16>, dim3((unsigned)M), dim3(256), 0, (hipStream_t)stream,
                           (const uint16_t*)A, K, Aq, alpha);
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}

size_t fq_gemm_w4a8_workspace_bytes(int64_t M, int64_t N, int64_t K, int group_size) {
    int g = 0;
    if (M <= 0 || w8_check(K, N, group_size, &g) != FQ_OK) return 0;
    const w8_plan p = w8_plan_of(M, N, K);
    return p.splits > 1 ? (size_t)p.splits * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
}

int fq_gemm_w4a8(const int8_t* Aq, const float* alpha, int64_t M, int64_t N, int64_t K, const void* codes,
                 const uint8_t* zscale, const void* tstep_f16, int group_size, void* C, int out_dtype,
                 void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0) return FQ_ERR_INVALID_ARG;
    if (out_dtype != FQ_F16 && out_dtype != FQ_BF16) return FQ_ERR_INVALID_ARG;
    int g = 0;
    const int st = w8_check(K, N, group_size, &g);
    if (st != FQ_OK) return st;
    if (M == 0) return FQ_OK;
    if (!Aq || !alpha || !codes || !zscale || !tstep_f16 || !C) return FQ_ERR_INVALID_ARG;
    if (M > (int64_t)1 << 24) return FQ_ERR_UNSUPPORTED;
    const size_t need = fq_gemm_w4a8_workspace_bytes(M, N, K, group_size);
    if (need > 0 && (!workspace || workspace_bytes < need)) return FQ_ERR_WORKSPACE;
    if (out_dtype == FQ_F16)
        return w8_gemm<FQ_F16>(Aq, alpha, M, N, K, codes, zscale, tstep_f16, g, C, workspace, (hipStream_t)stream);
    return w8_gemm<FQ_BF16>(Aq, alpha, M, N, K, codes, zscale, tstep_f16, g, C, workspace, (hipStream_t)stream);
}

}  // extern "C"
