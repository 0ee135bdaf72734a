// Packed code layout shared by the quantiser, the unpacker and the product kernels.
//
// The paper's kernels consume a pre-arranged weight buffer it does not describe
// (section 4.1 only notes that its block size of 64 equals the K extent of its kernel tile).  This layout is
// chosen for CDNA4: a wavefront's 64 lanes x 16 bytes is one contiguous KiB (eight full
// 128-byte lines), and the 16 bytes a lane receives are exactly the values it feeds, as
// they are, into v_mfma_f32_16x16x32 operands for one output column.
//
// Tile = 16 columns x KBLK rows, KBLK = 128 (3- and 4-bit) or 64 (8-bit), stored k-block-major:
//   codes[(kblock * (N / 16) + ntile) * 64 + lane] : 16 bytes
// with lane = j * 16 + (n % 16), j in 0..3.  All column tiles of one k-block are adjacent, so
// the waves that work on neighbouring columns at the same time read one contiguous stripe
// (like a plain streaming read), which keeps every HBM channel busy; a tile-major order
// would put concurrently read KiB a multiple of 32 KiB apart for the usual K.  Inside a tile, row k (0 <= k < KBLK) is
//   step t = k / 32, j = (k % 32) / 8, element e = k % 8
// i.e. MFMA step t contracts rows [32 t, 32 t + 32) and lane group j supplies 8
// consecutive rows of them.
//   4-bit: the lane's dword t holds the 8 elements of step t as nibbles; element e sits
//          at nibble position (e / 2) + 4 * (e % 2), so that masking with 0x000f000f
//          after a shift by 0/4/8/12 yields the element pairs (0,1), (2,3), (4,5), (6,7).
//          Stored nibble = q + 8 (1..15).
//   8-bit: the lane's bytes [8 t, 8 t + 8) hold elements 0..7 of step t.
//          Stored byte = q + 128 (1..255).
//   3-bit: a lane record is 12 bytes (three dwords) for the same 128 rows, records 12 bytes apart.
//          Dword t (t = 0, 1, 2) holds the elements of step t at the nibble positions of the 4-bit
//          form, each in the low three bits of its nibble: stored value = q + 4 (1..7).  The
//          fourth bit of every nibble carries step 3: bit 3 of nibble p of dword d is bit d of the
//          stored value of step 3's element at nibble position p.  Steps 0..2 are therefore usable
//          as they are (the conversion masks drop the fourth bit), and step 3 is three shifts and
//          masks away:  ((d0 >> 3) & 0x11111111) | ((d1 >> 2) & 0x22222222) | ((d2 >> 1) & 0x44444444).
#ifndef FQ_LAYOUT_H_
#define FQ_LAYOUT_H_

#include <stdint.h>

#define FQ_NTILE 16
#define FQ_KSTEP 32

__host__ __device__ constexpr int fq_kblk(int bits) { return bits == 8 ? 64 : 128; }
// bytes of one lane record
__host__ __device__ constexpr int fq_rec_bytes(int bits) { return bits == 3 ? 12 : 16; }

// Lane record that holds (k, n), and the position inside it.
struct fq_pos {
    int64_t rec;   // index of the lane record (16 bytes each; 12 for 3-bit codes)
    int t;         // MFMA step inside the k-block
    int e;         // element 0..7 inside the step
};

// Index of the lane record of (column tile, k-block, lane).
__host__ __device__ inline int64_t fq_rec(int64_t ntile, int64_t kb, int64_t ntiles, int lane) {
    return (kb * ntiles + ntile) * 64 + lane;
}

__host__ __device__ inline fq_pos fq_locate(int64_t k, int64_t n, int64_t N, int bits) {
    const int kblk = fq_kblk(bits);
    const int64_t ntile = n / FQ_NTILE;
    const int nl = (int)(n % FQ_NTILE);
    const int64_t kb = k / kblk;
    const int kr = (int)(k % kblk);
    fq_pos p;
    p.t = kr / FQ_KSTEP;
    const int j = (kr % FQ_KSTEP) / 8;
    p.e = kr % 8;
    p.rec = fq_rec(ntile, kb, N / FQ_NTILE, j * 16 + nl);
    return p;
}

__host__ __device__ inline int fq_nibble_slot(int e) { return (e >> 1) + 4 * (e & 1); }

// Stored value (q + 4) of a 3-bit code: d = the three dwords of its lane record.
__host__ __device__ inline uint32_t fq_get3(const uint32_t* d, int t, int e) {
    const int p = 4 * fq_nibble_slot(e);
    if (t < 3) return (d[t] >> p) & 7u;
    return ((d[0] >> (p + 3)) & 1u) | (((d[1] >> (p + 3)) & 1u) << 1) | (((d[2] >> (p + 3)) & 1u) << 2);
}
// The three dwords of a lane record from the stored values u[t][e] (t = 0..3, e = 0..7).
__host__ __device__ inline void fq_put3(const uint32_t (&u)[4][8], uint32_t* d) {
    d[0] = d[1] = d[2] = 0u;
    for (int e = 0; e < 8; ++e) {
        const int p = 4 * fq_nibble_slot(e);
        for (int t = 0; t < 3; ++t) d[t] |= (u[t][e] & 7u) << p;
        for (int b = 0; b < 3; ++b) d[b] |= ((u[3][e] >> b) & 1u) << (p + 3);
    }
}

#endif  // FQ_LAYOUT_H_
