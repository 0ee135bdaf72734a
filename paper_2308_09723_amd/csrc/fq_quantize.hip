// Quantiser, packer, unpacker and group-size heuristic kernels (gfx950).
//
// Appendix A: s = 2 max|w| / (2^b - 1), q = int(w / s); section 4.1: one scale per block
// of g consecutive rows of a column; Appendix B: scales stored in half precision.
// Rounding choices (scale rounded up to binary16, quotient in binary32, ties to even,
// clamp) are stated in fq.h.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "fq_internal.h"
#include "fq_layout.h"

namespace {

__device__ inline float half_bits_to_float(uint16_t b) {
    return __half2float(__ushort_as_half(b));
}

// stored scale (16 bits, binary16 or bfloat16) -> binary32
__device__ inline float scale_bits_to_float(uint16_t b, int sfmt) {
    return sfmt == FQ_SCALE_BF16 ? __uint_as_float((uint32_t)b << 16) : half_bits_to_float(b);
}

// Appendix A's scale for a group whose abs-max has the binary16 bit pattern m:
// the smallest s of the storage format with L * s >= 2 m (L = 2^bits - 1), as a 16-bit pattern.
// The candidate is the binary32 quotient rounded to nearest (binary16) or cut (bfloat16: at or
// below the quotient); the products L * candidate are exact in binary32 (8 x 11 bits at most),
// so one comparison decides whether the next value up is needed.
__device__ inline uint32_t scale_bits_from_absmax_bits(uint32_t m, float L, int sfmt) {
    const float two_m = 2.0f * half_bits_to_float((uint16_t)m);
    const float t32 = __fdiv_rn(two_m, L);
    uint32_t tb = sfmt == FQ_SCALE_BF16 ? (__float_as_uint(t32) >> 16)
                                        : (uint32_t)__half_as_ushort(__float2half_rn(t32));
    if (__fmul_rn(L, scale_bits_to_float((uint16_t)tb, sfmt)) < two_m) tb += 1;   // next value up
    return tb;
}

// ---------------------------------------------------------------------------------
// Scales: abs-max over each block of g rows, then the smallest storable s with
// L * s >= 2 m.  Block = 16 x 16 threads: thread (tx, ty) takes 8 consecutive columns (one
// 16-byte load per row, so a row of the block is 256 contiguous bytes) of the rows ty, ty + 16,
// ... of the group; the sixteen row slices are combined through LDS.
// ---------------------------------------------------------------------------------
typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));

// abs-max bit patterns of 8 columns (four packed pairs) over rows ty, ty + 16, ... < rows
__device__ inline uint4 absmax8_slice(const uint16_t* __restrict__ base, int64_t N, int rows, int ty) {
    u16x2_t m[4] = {{0, 0}, {0, 0}, {0, 0}, {0, 0}};
    auto fold = [&](const uint4& v) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t a = w[i] & 0x7fff7fffu;
            m[i] = __builtin_elementwise_max(m[i], __builtin_bit_cast(u16x2_t, a));
        }
    };
    int r = ty;
    for (; r + 48 < rows; r += 64) {      // four loads in flight
        const uint4 v0 = *reinterpret_cast<const uint4*>(base + (int64_t)r * N);
        const uint4 v1 = *reinterpret_cast<const uint4*>(base + (int64_t)(r + 16) * N);
        const uint4 v2 = *reinterpret_cast<const uint4*>(base + (int64_t)(r + 32) * N);
        const uint4 v3 = *reinterpret_cast<const uint4*>(base + (int64_t)(r + 48) * N);
        fold(v0); fold(v1); fold(v2); fold(v3);
    }
    for (; r < rows; r += 16) fold(*reinterpret_cast<const uint4*>(base + (int64_t)r * N));
    return make_uint4(__builtin_bit_cast(uint32_t, m[0]), __builtin_bit_cast(uint32_t, m[1]),
                      __builtin_bit_cast(uint32_t, m[2]), __builtin_bit_cast(uint32_t, m[3]));
}
// the sixteen slices of a block combined: valid in the threads with ty == 0
__device__ inline uint4 absmax8_block(uint4 mine, uint4 (&red)[16][16], int tx, int ty) {
    red[ty][tx] = mine;
    __syncthreads();
    if (ty != 0) return mine;
    u16x2_t m[4];
    m[0] = __builtin_bit_cast(u16x2_t, mine.x); m[1] = __builtin_bit_cast(u16x2_t, mine.y);
    m[2] = __builtin_bit_cast(u16x2_t, mine.z); m[3] = __builtin_bit_cast(u16x2_t, mine.w);
    for (int y = 1; y < 16; ++y) {
        const uint4 o = red[y][tx];
        m[0] = __builtin_elementwise_max(m[0], __builtin_bit_cast(u16x2_t, o.x));
        m[1] = __builtin_elementwise_max(m[1], __builtin_bit_cast(u16x2_t, o.y));
        m[2] = __builtin_elementwise_max(m[2], __builtin_bit_cast(u16x2_t, o.z));
        m[3] = __builtin_elementwise_max(m[3], __builtin_bit_cast(u16x2_t, o.w));
    }
    return make_uint4(__builtin_bit_cast(uint32_t, m[0]), __builtin_bit_cast(uint32_t, m[1]),
                      __builtin_bit_cast(uint32_t, m[2]), __builtin_bit_cast(uint32_t, m[3]));
}

__global__ __launch_bounds__(256) void fq_scales_kernel(const uint16_t* __restrict__ W, int64_t K,
                                                        int64_t N, int g, float L, int sfmt,
                                                        uint16_t* __restrict__ scales) {
    __shared__ uint4 red[16][16];
    const int tx = threadIdx.x, ty = threadIdx.y;
    const int64_t n = ((int64_t)blockIdx.x * 16 + tx) * 8;      // N is a multiple of 16
    const int64_t grp = blockIdx.y;
    uint4 m = make_uint4(0u, 0u, 0u, 0u);
    if (n < N) m = absmax8_slice(W + (grp * g) * N + n, N, g, ty);
    m = absmax8_block(m, red, tx, ty);
    if (ty == 0 && n < N) {
        const uint32_t w[4] = {m.x, m.y, m.z, m.w};
        uint32_t out[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            out[i] = scale_bits_from_absmax_bits(w[i] & 0xffffu, L, sfmt) |
                     (scale_bits_from_absmax_bits(w[i] >> 16, L, sfmt) << 16);
        *reinterpret_cast<uint4*>(scales + grp * N + n) = make_uint4(out[0], out[1], out[2], out[3]);
    }
}

// Coarse groups (few groups per column): the abs-max of 128-row blocks is taken first by
// fq_fine_absmax_kernel, with one block of threads per (128 rows x 128 columns), and this
// kernel folds the g / 128 block maxima of each group into its scale.  One kernel walking a
// whole 12288-row column per thread slice leaves most of the GPU idle.
__global__ __launch_bounds__(256) void fq_scales_fold_kernel(const uint16_t* __restrict__ fine, int64_t N,
                                                             int per_group, float L, int sfmt,
                                                             uint16_t* __restrict__ scales) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const int64_t grp = blockIdx.y;
    uint32_t m = 0;
    int i = 0;
    for (; i + 8 <= per_group; i += 8) {     // eight loads in flight
        uint32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = fine[(grp * per_group + i + u) * N + n];
#pragma unroll
        for (int u = 0; u < 8; ++u) m = v[u] > m ? v[u] : m;
    }
    for (; i < per_group; ++i) {
        const uint32_t v = fine[(grp * per_group + i) * N + n];
        m = v > m ? v : m;
    }
    scales[grp * N + n] = (uint16_t)scale_bits_from_absmax_bits(m, L, sfmt);
}

// ---------------------------------------------------------------------------------
// Encode: divide (IEEE binary32), round half to even, clamp (Appendix A's q = int(w / s)).
// ---------------------------------------------------------------------------------
// The quotient is formed without the division instruction sequence: with rs = 1 / s rounded to nearest
// (once per group; 0 for s = 0), x0 = w * rs is within two units in the last place of w / s, its residual
// e = w - x0 * s comes exactly out of one fused multiply-add, and x = x0 + e * rs (fused again) is the
// quotient rounded to nearest wherever that matters here: an exact tie k + 1/2 is representable and is
// returned exactly, and any other quotient of a binary16 weight by a binary16 or bfloat16 scale lies at
// least 2^-12 away from a tie (numerator and denominator are integers of at most 11 bits times powers of
// two), far beyond the error of x.  Checked on the host for every finite scale and every weight within
// the code range (tests/encode_identity_check.c: 2 x 10^9 pairs, no difference).  What the general
// division adds (scaling against overflow and subnormal quotients, the fix-ups for zero, infinity and
// NaN operands) cannot occur: |w / s| <= (2^bits - 1) / 2.
__device__ inline int encode_one(uint16_t wbits, float s, float rs, int qmax) {
    const float w = half_bits_to_float(wbits);
    const float x0 = w * rs;
    const float e = __builtin_fmaf(-x0, s, w);
    const float x = __builtin_fmaf(e, rs, x0);
    const float c = fminf(fmaxf(rintf(x), (float)-qmax), (float)qmax);
    return (int)c;
}

// ---------------------------------------------------------------------------------
// One-pass quantiser for group sizes that divide 128 (32, 64, 128): a block stages a panel of
// 128 rows x 128 columns of W in LDS with coalesced 16-byte loads, takes the abs-max of every
// 32-row sub-block, derives the scales of the panel's groups, and encodes and packs the panel
// from LDS.  W is read from HBM once (the two-pass path reads it twice, the second time with
// 2-byte loads).  Same arithmetic as the two-pass kernels, hence the same bits.
// ---------------------------------------------------------------------------------
#define FQ_QP_ROWS 128
#define FQ_QP_COLS 128
#define FQ_QP_PITCH (FQ_QP_COLS + 8)   // binary16 elements per LDS row
// OWN_SCALES = false: the scales were computed before (groups larger than the panel) and are only read.
template <int BITS, bool OWN_SCALES>
__global__ __launch_bounds__(256) void fq_quantize_panel_kernel(const uint16_t* __restrict__ W, int64_t K,
                                                                int64_t N, int g, float L, int sfmt,
                                                                uint16_t* __restrict__ scales,
                                                                uint32_t* __restrict__ codes) {
    constexpr int KBLK = fq_kblk(BITS);
    constexpr int STEPS = KBLK / FQ_KSTEP;
    constexpr int QMAX = (1 << (BITS - 1)) - 1;
    __shared__ uint16_t panel[FQ_QP_ROWS * FQ_QP_PITCH];
    __shared__ uint16_t submax[4][FQ_QP_COLS];      // abs-max bits of the 32-row sub-blocks
    __shared__ float sub_scale[4][FQ_QP_COLS];      // scale of the group each sub-block belongs to
    __shared__ float sub_rscale[4][FQ_QP_COLS];     // its reciprocal (0 for an all-zero group)
    const int tid = threadIdx.x;
    const int64_t n0 = (int64_t)blockIdx.x * FQ_QP_COLS;
    const int64_t k0 = (int64_t)blockIdx.y * FQ_QP_ROWS;
    const int cols = (int)((N - n0) < FQ_QP_COLS ? (N - n0) : FQ_QP_COLS);   // multiple of 16
    const int rows = (int)((K - k0) < FQ_QP_ROWS ? (K - k0) : FQ_QP_ROWS);   // 128, or 64 at the end (8-bit)

    // stage: thread -> (row = tid / 16 + 16 i, 8 columns starting at 8 (tid % 16))
    {
        const int c8 = (tid & 15) * 8;
#pragma unroll
        for (int i = 0; i < FQ_QP_ROWS / 16; ++i) {
            const int r = (tid >> 4) + 16 * i;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (r < rows && c8 < cols) v = *reinterpret_cast<const uint4*>(W + (k0 + r) * N + n0 + c8);
            *reinterpret_cast<uint4*>(&panel[r * FQ_QP_PITCH + c8]) = v;
        }
    }
    __syncthreads();
    if constexpr (OWN_SCALES) {
        // abs-max of the 32-row sub-blocks: thread -> column pair tid % 64, sub-block tid / 64; one 4-byte
        // LDS read per row and a packed 16-bit maximum
        {
            const int cp = (tid & 63) * 2;
            const int sb = tid >> 6;
            u16x2_t m = {0, 0};
#pragma unroll
            for (int r = 0; r < 32; ++r) {
                const uint32_t v = *reinterpret_cast<const uint32_t*>(&panel[(sb * 32 + r) * FQ_QP_PITCH + cp]);
                m = __builtin_elementwise_max(m, __builtin_bit_cast(u16x2_t, v & 0x7fff7fffu));
            }
            *reinterpret_cast<uint32_t*>(&submax[sb][cp]) = __builtin_bit_cast(uint32_t, m);
        }
        __syncthreads();
        // scales: one per (group, column); a group is g / 32 consecutive sub-blocks
        {
            const int per = g / 32;                 // 1, 2 or 4
            const int c = tid & 127;
    #pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int sb = (tid >> 7) + 2 * h;
                const int first = (sb / per) * per;
                uint32_t m = 0;
                for (int i = 0; i < per; ++i) {
                    const uint32_t a = submax[first + i][c];
                    m = a > m ? a : m;
                }
                const uint32_t sbits = scale_bits_from_absmax_bits(m, L, sfmt);
                const float sv = scale_bits_to_float((uint16_t)sbits, sfmt);
                sub_scale[sb][c] = sv;
                sub_rscale[sb][c] = sv == 0.0f ? 0.0f : __fdiv_rn(1.0f, sv);
                if (sb == first && sb * 32 < rows && c < cols) scales[((k0 + sb * 32) / g) * N + n0 + c] = (uint16_t)sbits;
            }
        }
        __syncthreads();
    } else {
        const int c = tid & 127;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int sb = (tid >> 7) + 2 * h;
            float v = 0.0f;
            if (sb * 32 < rows && c < cols) v = scale_bits_to_float(scales[((k0 + sb * 32) / g) * N + n0 + c], sfmt);
            sub_scale[sb][c] = v;
            sub_rscale[sb][c] = v == 0.0f ? 0.0f : __fdiv_rn(1.0f, v);
        }
        __syncthreads();
    }
    // encode + pack: wave w takes column tiles w, w + 4 of the panel
    const int lane = tid & 63, wave = tid >> 6;
    const int nl = lane & 15, j = lane >> 4;
    const int64_t ntiles = N / FQ_NTILE;
    for (int tl = wave; tl * FQ_NTILE < cols; tl += 4) {
        const int c = tl * FQ_NTILE + nl;
        for (int kb = 0; kb * KBLK < rows; ++kb) {
            uint32_t rec[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
                const int r0 = kb * KBLK + t * FQ_KSTEP + j * 8;
                const float sc = sub_scale[r0 / 32][c];
                const float rsc = sub_rscale[r0 / 32][c];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int q = encode_one(panel[(r0 + e) * FQ_QP_PITCH + c], sc, rsc, QMAX);
                    if (BITS == 4) {
                        rec[t] |= (uint32_t)(q + 8) << (4 * fq_nibble_slot(e));
                    } else if (BITS == 3) {
                        // steps 0..2: low three bits of the nibble; step 3: bit b of the value goes to
                        // the fourth bit of the same nibble of dword b
                        const uint32_t u = (uint32_t)(q + 4);
                        const int p = 4 * fq_nibble_slot(e);
                        if (t < 3) {
                            rec[t] |= u << p;
                        } else {
                            rec[0] |= (u & 1u) << (p + 3);
                            rec[1] |= ((u >> 1) & 1u) << (p + 3);
                            rec[2] |= ((u >> 2) & 1u) << (p + 3);
                        }
                    } else {
                        rec[2 * t + (e >> 2)] |= (uint32_t)(q + 128) << (8 * (e & 3));
                    }
                }
            }
            const int64_t kblock = (k0 / KBLK) + kb;
            const int64_t at = fq_rec(n0 / FQ_NTILE + tl, kblock, ntiles, lane);
            if (BITS == 3) {
                uint32_t* dst = codes + at * 3;
                dst[0] = rec[0];
                dst[1] = rec[1];
                dst[2] = rec[2];
            } else {
                *reinterpret_cast<uint4*>(codes + at * 4) = make_uint4(rec[0], rec[1], rec[2], rec[3]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// Unpack: one thread per logical element, writes are coalesced along N.
// ---------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(256) void fq_unpack_kernel(const uint32_t* __restrict__ codes, int64_t K,
                                                        int64_t N, int8_t* __restrict__ q) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    for (int64_t k = blockIdx.y; k < K; k += gridDim.y) {
        const fq_pos p = fq_locate(k, n, N, BITS);
        int v;
        if (BITS == 4) {
            const uint32_t w = codes[p.rec * 4 + p.t];
            v = (int)((w >> (4 * fq_nibble_slot(p.e))) & 0xfu) - 8;
        } else if (BITS == 3) {
            v = (int)fq_get3(codes + p.rec * 3, p.t, p.e) - 4;
        } else {
            const uint32_t w = codes[p.rec * 4 + 2 * p.t + (p.e >> 2)];
            v = (int)((w >> (8 * (p.e & 3))) & 0xffu) - 128;
        }
        q[k * N + n] = (int8_t)v;
    }
}

// ---------------------------------------------------------------------------------
// Heuristic (section 3.3).  Pass 1: abs-max of the finest blocks (f rows) -> fine[K/f, N]
// as binary16 bit patterns.  Pass 2: one thread per (column, coarsest group) folds the
// fine values pairwise, level by level, and sets flag[level] when the smaller child is
// below thr * parent.  The host then walks the flags from the coarsest level down.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fq_fine_absmax_kernel(const uint16_t* __restrict__ W, int64_t N,
                                                             int f, uint16_t* __restrict__ fine) {
    // thread layout as in fq_scales_kernel: 16 x 16, eight columns per thread
    __shared__ uint4 red[16][16];
    const int tx = threadIdx.x, ty = threadIdx.y;
    const int64_t n = ((int64_t)blockIdx.x * 16 + tx) * 8;
    const int64_t blk = blockIdx.y;
    uint4 m = make_uint4(0u, 0u, 0u, 0u);
    if (n < N) m = absmax8_slice(W + (blk * f) * N + n, N, f, ty);
    m = absmax8_block(m, red, tx, ty);
    if (ty == 0 && n < N) *reinterpret_cast<uint4*>(fine + blk * N + n) = m;
}

// levels = number of halvings covered; a top group spans 2^levels fine blocks.
// flag[l] (l = 0 is the coarsest transition g_start -> g_start/2) is set to 1 when any
// parent at that level has min(child) < thr * parent.
__global__ __launch_bounds__(256) void fq_halving_flags_kernel(const uint16_t* __restrict__ fine,
                                                               int64_t N, int64_t tops, int levels,
                                                               float thr, int* __restrict__ flags) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t top = blockIdx.y;
    if (n >= N || top >= tops) return;
    const int64_t span = (int64_t)1 << levels;
    const uint16_t* col = fine + (top * span) * N + n;
    // Level d = blockIdx.z (d = levels - 1 is the finest transition): parents are pairs of nodes of
    // 2^(levels-1-d) fine blocks, recomputed from the fine array, so a thread reads span values; one
    // grid layer per level keeps enough threads in flight when there are few top groups.
    const int d = blockIdx.z;
    const int64_t child = span >> (d + 1);     // fine blocks per child at this level
    bool hit = false;
    // one pass over the column's fine values (independent loads, several in flight): `node` collects the
    // child under way, `prev` is its left sibling once that one is complete
    uint32_t node = 0, prev = 0;
#pragma unroll 8
    for (int64_t q = 0; q < span; ++q) {
        const uint32_t a = col[q * N];
        node = a > node ? a : node;
        if (((q + 1) & (child - 1)) == 0) {            // a child ends here
            if (((q + 1) & (2 * child - 1)) == 0) {    // ... and it is the right one of its pair
                const float lo = half_bits_to_float((uint16_t)(prev < node ? prev : node));
                const float hi = half_bits_to_float((uint16_t)(prev < node ? node : prev));
                hit = hit || (lo < __fmul_rn(thr, hi));
            }
            prev = node;
            node = 0;
        }
    }
    if (hit) atomicOr(&flags[d], 1);
}

// The same test with the pairwise fold done in LDS (a top group of at most 1024 fine blocks): a block
// takes `cols` neighbouring columns of one top group, loads their 2^levels fine values with coalesced
// 4-byte loads, and folds them level by level from the finest transition up, alternating between two LDS
// arrays; every fine value is read from memory once instead of once per level, and no thread walks a
// whole column.  Dynamic LDS: 3 * 2^levels * cols bytes.
__global__ __launch_bounds__(256) void fq_halving_tree_kernel(const uint16_t* __restrict__ fine, int64_t N,
                                                              int levels, float thr, int cols,
                                                              int* __restrict__ flags) {
    extern __shared__ uint16_t tree[];     // [span][cols], then [span / 2][cols]
    const int tid = threadIdx.x;
    const int span = 1 << levels;
    const int64_t n0 = (int64_t)blockIdx.x * cols;
    const uint16_t* base = fine + ((int64_t)blockIdx.y * span) * N + n0;
    {
        const int pairs = cols / 2, c2 = (tid % pairs) * 2;
        const bool ok = n0 + c2 < N;       // N is even
        const int step = 256 / pairs;
        for (int r0 = tid / pairs; r0 < span; r0 += 8 * step) {     // eight loads in flight
            uint32_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = r0 + u * step;
                v[u] = (ok && r < span) ? *reinterpret_cast<const uint32_t*>(base + (int64_t)r * N + c2) : 0u;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = r0 + u * step;
                if (r < span) *reinterpret_cast<uint32_t*>(&tree[r * cols + c2]) = v[u];
            }
        }
    }
    __syncthreads();
    uint16_t* src = tree;
    uint16_t* dst = tree + span * cols;
    int len = span;                        // nodes per column at the level being folded
    const int lc = 31 - __clz(cols);       // cols is 16, 32 or 64
    for (int d = levels - 1; d >= 0; --d) {
        const int parents = len / 2;
        bool hit = false;
        for (int i = tid; i < parents * cols; i += 256) {
            const int p = i >> lc, c = i & (cols - 1);
            const uint32_t a = src[(2 * p) * cols + c], b = src[(2 * p + 1) * cols + c];
            const float lo = half_bits_to_float((uint16_t)(a < b ? a : b));
            const float hi = half_bits_to_float((uint16_t)(a < b ? b : a));
            hit = hit || (lo < __fmul_rn(thr, hi));
            dst[p * cols + c] = (uint16_t)(a < b ? b : a);
        }
        if (__syncthreads_or(hit) && tid == 0) atomicOr(&flags[d], 1);
        uint16_t* t = src;
        src = dst;
        dst = t;
        len = parents;
    }
}

__global__ void fq_zero_ints_kernel(int* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// ---------------------------------------------------------------------------------
// Round-trip error (section 3.2, figure 2a: mean squared error between the weights and their
// dequantised codes, Appendix A: dequantised value = q * s).  binary64 throughout: w, q * s and
// their difference are exact, the squares are rounded once, and the sums are taken in a fixed
// order (thread strip -> tree over the block -> one block over the per-block partials), so the
// result is deterministic.  part[0 .. nblk) holds the sums, part[nblk .. 2 nblk) the maxima.
// ---------------------------------------------------------------------------------
// A block takes a panel of 128 rows x 128 columns: the weights are staged in LDS with coalesced 16-byte loads,
// and every thread walks whole lane records of the packed codes (16 or 12 bytes, read in layout order: a wave
// reads one contiguous KiB) against the staged weights.  (Looking every weight's code up by its position
// instead reads the packed buffer four bytes at a time and computes a record address per weight.)
#define FQ_QE_PANEL 128
#define FQ_QE_PITCH 130   // binary16 elements per LDS row: rows 8 apart fall 8 banks apart
template <int BITS, bool EXACT32>
__global__ __launch_bounds__(256) void fq_quant_error_kernel(const uint16_t* __restrict__ W,
                                                             const uint32_t* __restrict__ codes,
                                                             const uint16_t* __restrict__ scales, int64_t K,
                                                             int64_t N, int g, int sfmt,
                                                             double* __restrict__ part, int64_t nblk) {
    __shared__ uint32_t wp[FQ_QE_PANEL * FQ_QE_PITCH / 2];
    __shared__ double sh_s[256];
    __shared__ double sh_m[256];
    constexpr int KBLK = fq_kblk(BITS);
    constexpr int STEPS = KBLK / FQ_KSTEP;
    constexpr int RW = fq_rec_bytes(BITS) / 4;                 // dwords per lane record
    constexpr int RECS = (FQ_QE_PANEL / KBLK) * (FQ_QE_PANEL / FQ_NTILE) * 64;
    const int tid = threadIdx.x;
    const int64_t panels_n = (N + FQ_QE_PANEL - 1) / FQ_QE_PANEL;
    const int64_t panels = panels_n * ((K + FQ_QE_PANEL - 1) / FQ_QE_PANEL);
    double sse = 0.0, mx = 0.0;
    float mxf = 0.0f;
    // With binary16 scales the error w - q s of one weight is formed in binary32, where it is exact: q s has at
    // most 19 significant bits, and when q != 0, |w| >= s / 2, so w, q s and their difference are multiples of
    // 2^(exponent of s - 11) below 2^(exponent of s + 8): 19 bits.  (q = 0: the error is w itself.)  Only its
    // square is accumulated in binary64; the largest magnitude is a binary32 maximum.  A third of the binary64
    // instructions per weight that the all-binary64 form needs, with the same bits in both results.
    // a block walks panels blockIdx.x, blockIdx.x + gridDim.x, ... (one partial result per block)
    for (int64_t pnl = blockIdx.x; pnl < panels; pnl += gridDim.x) {
    const int64_t n0 = (pnl % panels_n) * FQ_QE_PANEL;
    const int64_t k0 = (pnl / panels_n) * FQ_QE_PANEL;
    __syncthreads();                                           // the previous panel has been read
    for (int u = tid; u < FQ_QE_PANEL * 16; u += 256) {
        const int row = u >> 4, cu = u & 15;
        const int64_t k = k0 + row, n = n0 + cu * 8;
        if (k < K && n < N) {                                  // N is a multiple of 16: whole units
            const uint4 v = *reinterpret_cast<const uint4*>(W + k * N + n);
            uint32_t* dst = wp + row * (FQ_QE_PITCH / 2) + cu * 4;
            dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        }
    }
    __syncthreads();
    const uint16_t* wp16 = reinterpret_cast<const uint16_t*>(wp);
    for (int r = tid; r < RECS; r += 256) {
        const int lane = r & 63, tile_l = (r >> 6) & 7, kbl = r >> 9;
        const int col = tile_l * FQ_NTILE + (lane & 15);
        const int64_t n = n0 + col;
        const int64_t kb = k0 / KBLK + kbl;
        if (n >= N || kb * KBLK >= K) continue;
        const uint32_t* rec = codes + fq_rec(n / FQ_NTILE, kb, N / FQ_NTILE, lane) * RW;
        uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < RW; ++i) d[i] = rec[i];
        const int j = lane >> 4;
#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            const int krel = kbl * KBLK + FQ_KSTEP * t + 8 * j;
            const float sf = scale_bits_to_float(scales[((k0 + krel) / g) * N + n], sfmt);
            const double sv = (double)sf;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int q;
                if (BITS == 4) q = (int)((d[t] >> (4 * fq_nibble_slot(e))) & 0xfu) - 8;
                else if (BITS == 3) q = (int)fq_get3(d, t, e) - 4;
                else q = (int)((d[2 * t + (e >> 2)] >> (8 * (e & 3))) & 0xffu) - 128;
                const float wf = half_bits_to_float(wp16[(krel + e) * FQ_QE_PITCH + col]);
                if constexpr (EXACT32) {
                    const float ef = __builtin_fmaf(-(float)q, sf, wf);
                    const double err = (double)ef;
                    sse += err * err;
                    mxf = fmaxf(mxf, fabsf(ef));
                } else {
                    const double err = (double)wf - (double)q * sv;
                    sse += err * err;
                    mx = fmax(mx, fabs(err));
                }
            }
        }
    }
    }
    sh_s[tid] = sse;
    sh_m[tid] = fmax(mx, (double)mxf);
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (tid < w) {
            sh_s[tid] += sh_s[tid + w];
            sh_m[tid] = fmax(sh_m[tid], sh_m[tid + w]);
        }
        __syncthreads();
    }
    if (tid == 0) {
        part[blockIdx.x] = sh_s[0];
        part[nblk + blockIdx.x] = sh_m[0];
    }
}

__global__ __launch_bounds__(256) void fq_quant_error_final_kernel(const double* __restrict__ part, int64_t nblk,
                                                                   double* __restrict__ out) {
    __shared__ double sh_s[256];
    __shared__ double sh_m[256];
    double sse = 0.0, mx = 0.0;
    for (int64_t i = threadIdx.x; i < nblk; i += 256) {
        sse += part[i];
        mx = fmax(mx, part[nblk + i]);
    }
    sh_s[threadIdx.x] = sse;
    sh_m[threadIdx.x] = mx;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            sh_s[threadIdx.x] += sh_s[threadIdx.x + w];
            sh_m[threadIdx.x] = fmax(sh_m[threadIdx.x], sh_m[threadIdx.x + w]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        out[0] = sh_s[0];
        out[1] = sh_m[0];
    }
}

}  // namespace

// ---------------------------------------------------------------------------------
// Measurement helper: reads a buffer and nothing else (16 bytes per lane, four non-temporal loads in
// flight per lane, grid-stride), one checksum word per block so that the loads cannot be dropped.
// Launched as 256 blocks of 768 threads, the shape of the small-M product kernel; of the shapes tried
// (256 ... 2048 blocks of 256 ... 1024 threads, 2 ... 8 loads in flight) this is among the fastest
// (7.1 - 7.3 TB/s), whereas grids whose stride between a lane's loads is 4 or 8 MiB lose 15 - 20 %, and
// ordinary (temporal) loads 10 %.
// ---------------------------------------------------------------------------------
typedef uint32_t probe_u32x4 __attribute__((ext_vector_type(4)));
#define FQ_PROBE_BLOCKS 256
#define FQ_PROBE_THREADS 768
__global__ __launch_bounds__(FQ_PROBE_THREADS) void fq_stream_read_kernel(const probe_u32x4* __restrict__ buf,
                                                                          size_t units,
                                                                          uint32_t* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * FQ_PROBE_THREADS;
    size_t i = (size_t)blockIdx.x * FQ_PROBE_THREADS + threadIdx.x;
    probe_u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 3 * stride < units; i += 4 * stride) {
        const probe_u32x4 a = __builtin_nontemporal_load(buf + i);
        const probe_u32x4 b = __builtin_nontemporal_load(buf + i + stride);
        const probe_u32x4 c = __builtin_nontemporal_load(buf + i + 2 * stride);
        const probe_u32x4 d = __builtin_nontemporal_load(buf + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < units; i += stride) acc ^= __builtin_nontemporal_load(buf + i);
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x ^= (uint32_t)__shfl_xor((int)x, o, 64);
    __shared__ uint32_t red[FQ_PROBE_THREADS / 64];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t y = 0;
        for (int w = 0; w < FQ_PROBE_THREADS / 64; ++w) y ^= red[w];
        sink[blockIdx.x] = y;
    }
}

// ----------------------------------------------------------------------------- launchers
int fq_launch_stream_read_probe(const void* buf, size_t bytes, void* sink, hipStream_t stream) {
    hipLaunchKernelGGL(fq_stream_read_kernel, dim3(FQ_PROBE_BLOCKS), dim3(FQ_PROBE_THREADS), 0, stream, (const probe_u32x4*)buf, bytes / 16,
                       (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}

#define FQ_LAUNCH_PANEL(OWN)                                                                                  \
    do {                                                                                                      \
        if (bits == 3)                                                                                        \
            hipLaunchKernelGGL((fq_quantize_panel_kernel<3, OWN>), grid, dim3(256), 0, stream,                \
                               (const uint16_t*)W, K, N, g, L, sfmt, (uint16_t*)scales, (uint32_t*)codes);    \
        else if (bits == 4)                                                                                   \
            hipLaunchKernelGGL((fq_quantize_panel_kernel<4, OWN>), grid, dim3(256), 0, stream,                \
                               (const uint16_t*)W, K, N, g, L, sfmt, (uint16_t*)scales, (uint32_t*)codes);    \
        else                                                                                                  \
            hipLaunchKernelGGL((fq_quantize_panel_kernel<8, OWN>), grid, dim3(256), 0, stream,                \
                               (const uint16_t*)W, K, N, g, L, sfmt, (uint16_t*)scales, (uint32_t*)codes);    \
    } while (0)

int fq_launch_quantize(const void* W, int64_t K, int64_t N, int bits, int g, int sfmt, void* codes, void* scales,
                       hipStream_t stream) {
    const float L = (float)((1 << bits) - 1);
    if (g == 32 || g == 64 || g == 128) {
        dim3 grid((unsigned)((N + FQ_QP_COLS - 1) / FQ_QP_COLS), (unsigned)((K + FQ_QP_ROWS - 1) / FQ_QP_ROWS));
        FQ_LAUNCH_PANEL(true);
        return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
    }
    if (g >= 1024 && g % 128 == 0) {
        // two stages; the block maxima (K / 128 x N binary16 = K * N / 64 bytes) are parked in the
        // code buffer, which is only written by the encoding pass below
        uint16_t* fine = (uint16_t*)codes;
        dim3 block(16, 16);
        dim3 grid((unsigned)((N + 127) / 128), (unsigned)(K / 128));
        hipLaunchKernelGGL(fq_fine_absmax_kernel, grid, block, 0, stream, (const uint16_t*)W, N, 128, fine);
        dim3 grid2((unsigned)((N + 255) / 256), (unsigned)(K / g));
        hipLaunchKernelGGL(fq_scales_fold_kernel, grid2, dim3(256), 0, stream, (const uint16_t*)fine, N, g / 128, L,
                           sfmt, (uint16_t*)scales);
    } else {
        dim3 block(16, 16);
        dim3 grid((unsigned)((N + 127) / 128), (unsigned)(K / g));
        hipLaunchKernelGGL(fq_scales_kernel, grid, block, 0, stream, (const uint16_t*)W, K, N, g, L, sfmt,
                           (uint16_t*)scales);
    }
    {
        // encoding pass from LDS panels, with the scales just written
        dim3 grid((unsigned)((N + FQ_QP_COLS - 1) / FQ_QP_COLS), (unsigned)((K + FQ_QP_ROWS - 1) / FQ_QP_ROWS));
        FQ_LAUNCH_PANEL(false);
    }
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}

int fq_launch_unpack(const void* codes, int64_t K, int64_t N, int bits, int8_t* q, hipStream_t stream) {
    dim3 block(256);
    dim3 grid((unsigned)((N + 255) / 256), (unsigned)(K < 16384 ? K : 16384));
    if (bits == 3)
        hipLaunchKernelGGL(fq_unpack_kernel<3>, grid, block, 0, stream, (const uint32_t*)codes, K, N, q);
    else if (bits == 4)
        hipLaunchKernelGGL(fq_unpack_kernel<4>, grid, block, 0, stream, (const uint32_t*)codes, K, N, q);
    else
        hipLaunchKernelGGL(fq_unpack_kernel<8>, grid, block, 0, stream, (const uint32_t*)codes, K, N, q);
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}

int fq_launch_choose_group(const void* W, int64_t K, int64_t N, int g_top, int levels, float alpha,
                           int* flags_host, void* workspace, hipStream_t stream) {
    // workspace: [flags: 64 ints][fine: (K / f) * N binary16]
    int* flags = (int*)workspace;
    uint16_t* fine = (uint16_t*)((char*)workspace + 256);
    const int f = g_top >> levels;
    hipLaunchKernelGGL(fq_zero_ints_kernel, dim3(1), dim3(64), 0, stream, flags, 64);
    {
        dim3 block(16, 16);
        dim3 grid((unsigned)((N + 127) / 128), (unsigned)(K / f));
        hipLaunchKernelGGL(fq_fine_absmax_kernel, grid, block, 0, stream, (const uint16_t*)W, N, f, fine);
    }
    {
        const float thr = 1.0f - alpha;
        if (levels <= 10) {
            // fold in LDS: 64 / 32 / 16 columns per block for up to 256 / 512 / 1024 fine blocks (<= 48 KiB)
            const int cols = levels <= 8 ? 64 : (levels == 9 ? 32 : 16);
            dim3 grid((unsigned)((N + cols - 1) / cols), (unsigned)(K / g_top));
            hipLaunchKernelGGL(fq_halving_tree_kernel, grid, dim3(256), (size_t)3 * ((size_t)1 << levels) * cols,
                               stream, (const uint16_t*)fine, N, levels, thr, cols, flags);
        } else {
            dim3 block(256);
            dim3 grid((unsigned)((N + 255) / 256), (unsigned)(K / g_top), (unsigned)levels);   // levels >= 1
            hipLaunchKernelGGL(fq_halving_flags_kernel, grid, block, 0, stream, (const uint16_t*)fine, N,
                               K / g_top, levels, thr, flags);
        }
    }
    if (hipGetLastError() != hipSuccess) return FQ_ERR_HIP;
    if (hipMemcpyAsync(flags_host, flags, sizeof(int) * 64, hipMemcpyDeviceToHost, stream) != hipSuccess)
        return FQ_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return FQ_ERR_HIP;
    return FQ_OK;
}

int64_t fq_quant_error_blocks(int64_t K, int64_t N) {
    const int64_t panels = ((N + FQ_QE_PANEL - 1) / FQ_QE_PANEL) * ((K + FQ_QE_PANEL - 1) / FQ_QE_PANEL);
    return panels < 2048 ? panels : 2048;
}

int fq_launch_quant_error(const void* W, int64_t K, int64_t N, int bits, int g, int sfmt, const void* codes,
                          const void* scales, double* out_host2, void* workspace, hipStream_t stream) {
    // workspace: [out: 2 doubles][partials: 2 * nblk doubles]
    double* out = (double*)workspace;
    double* part = out + 2;
    const int64_t nblk = fq_quant_error_blocks(K, N);
    dim3 grid((unsigned)nblk);
#define FQ_QE_GO(B_, X_)                                                                                    \
    hipLaunchKernelGGL((fq_quant_error_kernel<B_, X_>), grid, dim3(256), 0, stream, (const uint16_t*)W,     \
                       (const uint32_t*)codes, (const uint16_t*)scales, K, N, g, sfmt, part, nblk)
    const bool x32 = sfmt == FQ_SCALE_F16;
    if (bits == 3) { if (x32) FQ_QE_GO(3, true); else FQ_QE_GO(3, false); }
    else if (bits == 4) { if (x32) FQ_QE_GO(4, true); else FQ_QE_GO(4, false); }
    else { if (x32) FQ_QE_GO(8, true); else FQ_QE_GO(8, false); }
#undef FQ_QE_GO
    hipLaunchKernelGGL(fq_quant_error_final_kernel, dim3(1), dim3(256), 0, stream, (const double*)part, nblk, out);
    if (hipGetLastError() != hipSuccess) return FQ_ERR_HIP;
    if (hipMemcpyAsync(out_host2, out, sizeof(double) * 2, hipMemcpyDeviceToHost, stream) != hipSuccess)
        return FQ_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return FQ_ERR_HIP;
    return FQ_OK;
}
