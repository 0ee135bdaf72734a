// Packed code layout shared by the quantiser, the unpacker and the product kernels.
//
// The paper's kernels consume a pre-arranged weight buffer it does not describe
// (section 4.1 only says the block size 64 "matches the K tile size").  This layout is
// chosen for CDNA4: a wavefront's 64 lanes x 16 bytes is one contiguous KiB (eight full
// 128-byte lines), and the 16 bytes a lane receives are exactly the values it feeds, as
// they are, into v_mfma_f32_16x16x32 operands for one output column.
//
// Tile = 16 columns x KBLK rows, KBLK = 128 (4-bit) or 64 (8-bit), stored k-block-major:
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
#ifndef FQ_LAYOUT_H_
#define FQ_LAYOUT_H_

#include <stdint.h>

#define FQ_NTILE 16
#define FQ_KSTEP 32

__host__ __device__ constexpr int fq_kblk(int bits) { return bits == 4 ? 128 : 64; }

// Byte offset of the 16-byte lane record that holds (k, n), and the position inside it.
struct fq_pos {
    int64_t rec;   // index of the 16-byte record
    int t;         // MFMA step inside the k-block
    int e;         // element 0..7 inside the step
};

// Index of the 16-byte record of (column tile, k-block, lane).
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

#endif  // FQ_LAYOUT_H_
