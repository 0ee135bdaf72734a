// Host side of the product: the plan (which kernel, which block shape) and the entry points
// that dispatch on activation type and code width.  The kernels themselves are instantiated
// in fq_gemm_<type>_<bits>.hip.
#include <hip/hip_runtime.h>
#include <math.h>
#include <mutex>
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
                                               void* C, const hipStream_t* streams);
FQ_DECLARE_GEMM(0, 4)
FQ_DECLARE_GEMM(0, 8)
FQ_DECLARE_GEMM(1, 4)
FQ_DECLARE_GEMM(1, 8)
FQ_DECLARE_GEMM(2, 4)   // bf16 activations, bf16 scales
FQ_DECLARE_GEMM(2, 8)
FQ_DECLARE_GEMM(0, 3)   // 3-bit codes
FQ_DECLARE_GEMM(1, 3)
FQ_DECLARE_GEMM(2, 3)

// Compute units of the device, asked once per process (the current device at the first call); without a
// device (host-only use of the size queries and fq_gemm_describe) the MI355X's 256.
int fq_cu_count() {
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            return v;
        (void)hipGetLastError();
        return 256;
    }();
    return n;
}

fq_gemm_plan fq_plan_gemm(int64_t M, int64_t N, int64_t K, int bits, int g) {
    fq_gemm_plan p = {};
    const int ncu = fq_cu_count();
    const int kblk = fq_kblk(bits);
    const int KB = (int)(K / kblk);
    const int ntiles = (int)(N / FQ_NTILE);
    if (M <= 16) {
        // One block per compute unit, all resident at once.  Candidates are scored by how evenly
        // the column tiles (times the grid's split of K) fill one block per compute unit, by the bytes a compute
        // unit keeps in flight (waves x NT KiB x ring depth, ~64 KiB saturates), and by how many
        // activation units a lane must stage (fewer registers); ties keep the earlier variant.
        // The factors come from sweeps over the OPT-175B shapes at M = 1 and 8.
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
                const int need = (int)M * kc;
                const int au = need <= 64 * gp ? 1 : (need <= 128 * gp ? 2 : (need <= 256 * gp ? 4 : 0));
                if (au == 0) continue;
                // (all the waves the register class allows: with one column group per block, twelve k-workers
                // of two stages measured 3 - 8 % faster than eight of three on the 12288-column layers)
                int kw = sv.maxw / gp;
                if (kw > KB) kw = KB;
                if (kw < 1) continue;
                const int SB = (KB + kw - 1) / kw;       // iterations if one block walks all of K
                // Few column blocks: K is also split over the grid (binary32 partials + a second kernel),
                // which moreover divides the activation bytes every block has to fetch.
                int gs = 1;
                if (blocks <= ncu / 2) gs = (int)(ncu / blocks);
                if (gs > 8) gs = 8;
                if (gs > SB) gs = SB;
                const int64_t grid = blocks * gs;
                const int64_t rounds = (grid + ncu - 1) / ncu;
                const double eff = (double)ntiles * gs / (double)(rounds * ncu * tb);
                const int waves = gp * kw;
                const double inflight = (double)waves * sv.nt * sv.depth;   // KiB
                const double n_it = (double)((SB + gs - 1) / gs);
                double score = eff * eff * (inflight >= 64.0 ? 1.0 : sqrt(inflight / 64.0)) * f_nt[sv.nt];
                score /= 1.0 + 0.1 * (double)(rounds - 1);   // a single resident round beats several
                score *= au == 1 ? 1.0 : (au == 2 ? 0.8 : 0.6);
                // a split of K over the grid costs a second kernel, and with few iterations left per
                // block the register ring is mostly filling and draining
                if (gs > 1) score *= n_it >= 16.0 ? 0.80 : 0.65;
                // every block fetches its whole k range of the activations: M * K * 2 / gs bytes,
                // once per block, next to K * N * bits / 8 bytes of weights
                score /= 1.0 + 0.15 * ((double)M * 2.0 * (double)ncu / gs) / ((double)N * bits / 8.0);
                if (waves < 6) score *= 0.85;
                if (kw == 1) score *= 0.95;                  // no k-workers: measured ~5 % slower
                if (score > best + 1e-9) {
                    best = score;
                    p.variant = v;
                    p.gp = gp;
                    p.kw = kw;
                    p.au = au;
                    p.waves = waves;
                    p.splits = gs;
                }
            }
        }
        p.kb_per_split = 0;
    } else {
        // Tiled MFMA kernel: BM = 16 * mt rows per block (mt = 2, 4 or 8), 48 columns per wave, 4 or 8
        // waves, and optionally a split of K over `splits` blocks whose binary32 partial tiles a second
        // kernel adds.  The block shape is the one that minimises a measured cost model:
        //   time = ceil(blocks / compute units) * k-blocks per block * u(mt, waves)  +  cost of the partials
        // where u is the time one block spends on one k-block of 128 rows of K when every compute
        // unit holds its share of blocks (microseconds), and the partials cost their write plus read
        // at ~5 TB/s plus a launch.  The constants are a least-squares fit (of log time; rms error
        // 9 - 11 %) to exhaustive sweeps of (mt, waves, splits) over the OPT-175B shapes at M = 17 ...
        // 256, both activation types, separately for the four kinds of kernels the dispatch
        // distinguishes (4-bit codes with 1, 2 or 4 scale rows per k-block, of which only the first
        // runs post-scaled at every small shape; 8-bit codes): the model's choice is 0.5 - 2 % slower
        // than the sweep's best on average, 15 % at worst.
        // Up to 256 rows the smaller blocks compete with the 128-row ones (several row blocks, each
        // converting the weights again) and often win there, e.g. QKV at M = 128 in two 64-row blocks
        // and no split of K; beyond 256 rows only the 128-row shapes are candidates.
        p.kind = 1;
        //   u8(mt=2) u4(mt=2) u8(mt=4) u4(mt=4) u8(mt=8) u4(mt=8)  lone 4-wave block factor (mt < 8, mt = 8)
        static const double consts[4][8] = {
            {0.99, 0.506, 1.43, 0.83, 2.33, 1.43, 1.2, 1.2},     // 4-bit, one scale row per k-block
            {1.17, 0.634, 1.60, 0.884, 2.34, 1.46, 1.2, 1.2},    // 4-bit, two scale rows
            {1.64, 0.731, 2.16, 1.29, 2.70, 1.57, 1.5, 1.35},    // 4-bit, four scale rows
            {1.73, 0.77, 1.73, 1.035, 2.50, 1.47, 1.2, 1.35}};   // 8-bit
        const int sr4 = g % 128 == 0 ? 1 : (128 % g == 0 ? 128 / g : 4);
        const double* cs = consts[bits == 8 ? 3 : (sr4 == 1 ? 0 : (sr4 == 2 ? 1 : 2))];
        const int split_opts[6] = {1, 2, 3, 4, 6, 8};
        double best = 1e30;
        p.tail_tiles = 0;
        p.tail_splits = 1;
        p.tail_kbs = 0;
        for (int mt = 8; mt >= 2; mt /= 2) {
            // a block shape is a candidate when the matrix has more rows than half its height (the
            // smallest always is), and the small ones only up to 256 rows
            if (mt > 2 && (int64_t)mt * 8 >= M) continue;
            if (mt < 8 && M > 256) continue;
            const int bm = mt * 16;
            const int64_t nbm = (M + bm - 1) / bm;
            const double u8 = mt == 8 ? cs[4] : (mt == 4 ? cs[2] : cs[0]);
            const double u4 = mt == 8 ? cs[5] : (mt == 4 ? cs[3] : cs[1]);
            for (int waves = 8; waves >= 4; waves -= 4) {
                const int64_t nbn = (ntiles + waves * MMA_NT - 1) / (waves * MMA_NT);
                // k-blocks of this shape: 8-bit codes in the 128-row, 8-wave shape go two layout blocks at
                // a time (measured ~7 % less per row of K)
                const int kblk_c = fq_mma_kblk(bits, mt, waves, K, g);
                const int KB = (int)(K / kblk_c);
                const double kscale = (double)kblk_c / 128.0 * (kblk_c != kblk ? 0.93 : 1.0);
                const double u = (waves == 8 ? u8 : u4) * kscale;
                for (int si = 0; si < 6; ++si) {
                    int splits = split_opts[si];
                    if (splits > KB) break;
                    const int kbs = (KB + splits - 1) / splits;
                    splits = (KB + kbs - 1) / kbs;
                    const int64_t blocks = nbn * nbm * splits;
                    const int64_t per_cu = (blocks + ncu - 1) / ncu;
                    double t = (double)per_cu * kbs * u;
                    if (waves == 4) {
                        // u is a 4-wave block's share when `cap` of them run together on a compute unit; the
                        // ones left over run with idle SIMDs and take longer than that share
                        const int cap = mt == 2 ? 3 : 2;
                        const int64_t left = per_cu % cap;
                        if (left > 0) {
                            const double f = per_cu < cap ? (mt == 8 ? cs[7] : cs[6]) : (mt == 8 ? 1.13 : 1.0);
                            t += (f - 1.0) * (double)left * kbs * u;
                        }
                    }
                    // (with fewer blocks than compute units a block takes as long as in a full grid)
                    if (splits > 1) t += 2.0 * splits * (double)M * (double)N * 4.0 / 5e6 + 5.0;
                    if (t < best - 1e-9) {
                        best = t;
                        p.mt = mt;
                        p.waves = waves;
                        p.splits = splits;
                        p.kb_per_split = kbs;
                        p.tail_tiles = 0;
                        p.tail_splits = 1;
                        p.tail_kbs = 0;
                    }
                }
                // No uniform split, but the tiles of the partly filled last round are split along K so
                // that they occupy every block slot once more: the last round then lasts 1 / tail_splits
                // of a full one, at the price of partial tiles for those tiles only.
                const int64_t tiles = nbn * nbm;
                const int64_t slots = (int64_t)ncu * (waves == 8 ? 1 : (mt == 2 ? 3 : 2));
                const int64_t rem = tiles % slots;
                if (tiles > slots && rem > 0) {
                    int ts = (int)(slots / rem);
                    if (ts > 8) ts = 8;
                    if (ts > KB) ts = KB;
                    if (ts >= 2) {
                        const int tkbs = (KB + ts - 1) / ts;
                        ts = (KB + tkbs - 1) / tkbs;
                        const int64_t head = tiles - rem;
                        double t = (double)(head / ncu) * KB * u + (double)((rem * ts + ncu - 1) / ncu) * tkbs * u;
                        const double bm_bn = (double)bm * (double)(waves * MMA_NT * FQ_NTILE);
                        t += 2.0 * ts * (double)rem * bm_bn * 4.0 / 5e6 + 5.0;
                        // for the small shapes the model is 10 % optimistic about this form (QKV at M = 256:
                        // 221 us predicted, 244 measured), so it has to win by that much
                        if (mt < 8) t *= 1.10;
                        if (ts >= 2 && t < best - 1e-9) {
                            best = t;
                            p.mt = mt;
                            p.waves = waves;
                            p.splits = 1;
                            p.kb_per_split = KB;
                            p.tail_tiles = (int)rem;
                            p.tail_splits = ts;
                            p.tail_kbs = tkbs;
                        }
                    }
                }
            }
        }
    }
    return p;
}

int fq_launch_gemm(const void* A, int act, int64_t M, int64_t N, int64_t K, const void* codes,
                   const void* scales, int bits, int g, void* C, void* workspace, hipStream_t stream) {
    const fq_gemm_plan plan = fq_plan_gemm(M, N, K, bits, g);
#define FQ_PICK(ACT)                                                                                        \
    (bits == 3   ? fq_launch_typed_##ACT##_3(A, M, N, K, codes, scales, g, C, workspace, plan, stream)      \
     : bits == 4 ? fq_launch_typed_##ACT##_4(A, M, N, K, codes, scales, g, C, workspace, plan, stream)      \
                 : fq_launch_typed_##ACT##_8(A, M, N, K, codes, scales, g, C, workspace, plan, stream))
    if (act == FQ_F16) return FQ_PICK(0);
    if (act == FQ_BF16) return FQ_PICK(1);
    return FQ_PICK(2);
#undef FQ_PICK
}

// The grouped product launches up to three kernels (row tiles of 128, 64 and 32 rows) that do not
// depend on each other.  Launched one after the other on the caller's stream, each would end with
// a partly filled last round of blocks; on three streams the blocks of the next kernel fill the
// compute units the previous one leaves idle.  The two extra streams (default priority) and the
// events that fork them from and join them to the caller's stream are created once per device and
// live until the process ends.
namespace {
struct fq_side {
    bool tried = false, ok = false;
    hipStream_t s[2];
    hipEvent_t fork, join[2];
};
std::mutex g_side_mutex;    // guards the creation of the side streams
std::mutex g_fork_mutex;    // serialises fork ... join sequences: the events are shared by all callers on a device
fq_side g_side[64];

fq_side* side_streams() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(g_side_mutex);
    fq_side& x = g_side[dev];
    if (!x.tried) {
        x.tried = true;
        bool ok = hipStreamCreateWithFlags(&x.s[0], hipStreamNonBlocking) == hipSuccess &&
                  hipStreamCreateWithFlags(&x.s[1], hipStreamNonBlocking) == hipSuccess &&
                  hipEventCreateWithFlags(&x.fork, hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&x.join[0], hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&x.join[1], hipEventDisableTiming) == hipSuccess;
        x.ok = ok;
        if (!ok) (void)hipGetLastError();
    }
    return x.ok ? &x : nullptr;
}
}  // namespace

int fq_launch_gemm_grouped(const void* A, int act, const int32_t* offsets, int E, int64_t N, int64_t K,
                           const void* codes, const void* scales, int bits, int g, void* C,
                           hipStream_t stream) {
    // which tile sizes occur (same cutting rule as the launcher)
    bool has[3] = {false, false, false};
    for (int e = 0; e < E; ++e) {
        const int32_t rows = offsets[e + 1] - offsets[e];
        if (rows <= 0) continue;
        if (rows > 64) has[0] = true;
        const int32_t rest = rows > 64 ? rows % 128 : rows;
        if (rest > 64) has[0] = true;
        else if (rest > 32) has[1] = true;
        else if (rest > 0) has[2] = true;
    }
    hipStream_t streams[3] = {stream, stream, stream};
    fq_side* side = (int)has[0] + (int)has[1] + (int)has[2] > 1 ? side_streams() : nullptr;
    // host threads that fork at the same time would record and wait on each other's events
    std::unique_lock<std::mutex> fork_lock(g_fork_mutex, std::defer_lock);
    if (side) fork_lock.lock();
    bool forked[2] = {false, false};
    if (side) {
        // the first tile size present stays on the caller's stream, the others go to the side streams
        int next = 0;
        bool first = true;
        if (hipEventRecord(side->fork, stream) != hipSuccess) return FQ_ERR_HIP;
        for (int c = 0; c < 3; ++c) {
            if (!has[c]) continue;
            if (first) { first = false; continue; }
            if (hipStreamWaitEvent(side->s[next], side->fork, 0) != hipSuccess) return FQ_ERR_HIP;
            streams[c] = side->s[next];
            forked[next] = true;
            ++next;
        }
    }
    int st;
#define FQ_PICK(ACT)                                                                                        \
    (bits == 3   ? fq_launch_grouped_typed_##ACT##_3(A, offsets, E, N, K, codes, scales, g, C, streams)     \
     : bits == 4 ? fq_launch_grouped_typed_##ACT##_4(A, offsets, E, N, K, codes, scales, g, C, streams)     \
                 : fq_launch_grouped_typed_##ACT##_8(A, offsets, E, N, K, codes, scales, g, C, streams))
    if (act == FQ_F16) st = FQ_PICK(0);
    else if (act == FQ_BF16) st = FQ_PICK(1);
    else st = FQ_PICK(2);
#undef FQ_PICK
    // join even after a failed launch, so that the side streams never run ahead of the caller's
    for (int i = 0; i < 2; ++i) {
        if (!forked[i]) continue;
        if (hipEventRecord(side->join[i], side->s[i]) != hipSuccess ||
            hipStreamWaitEvent(stream, side->join[i], 0) != hipSuccess)
            st = st == FQ_OK ? FQ_ERR_HIP : st;
    }
    return st;
}
