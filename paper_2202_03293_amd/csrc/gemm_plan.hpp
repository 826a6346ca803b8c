// Host side of the GEMM kernels: the argument block both kernels take, the table of compiled tiles
// (gemm_kernel.hpp instantiates them in this order), the plan of one launch, and the cost model that
// picks tile, k-split or the register-direct kernel (gemm_direct.hip) for a shape.  No device code
// here.
#pragma once
#include "lg_common.hpp"

namespace lg {

struct ConvGeom {        // implicit-GEMM A operand: row m -> (n, oh, ow), column k -> (kh, kw, c)
    int64_t H, W, C, KW, SH, SW, DH, DW, OH, OW;
};

struct GemmArgs {
    const float* A;      // AB, A B^T: M x K (row stride lda).  A^T B: K x M.  conv: NHWC input
    const float* B;      // AB, A^T B: K x N (row stride ldb).  A B^T: N x K
    float* C;            // M x N, row stride ldc (or split-k partials: slab z at C + z*M*ldc)
    int64_t M, N, K;
    int64_t lda, ldb, ldc;
    int64_t k_per_split; // multiple of the tile's BK; slab z covers k in [z*k_per_split, min(K, (z+1)*k_per_split))
    int accumulate;      // only honoured when the grid has one k-slab
    unsigned tiles_m, tiles_n;
    ConvGeom g;
};

enum class Layout { NN, CONV, TN, NT };

// The register-direct kernel for small and skinny problems (gemm_direct.hip); returns an LG_* status.
int launch_direct(const GemmArgs& a, Layout layout, int nbw, int ks, hipStream_t s);
bool direct_can_run(const GemmArgs& a, Layout layout);     // operands within its 32-bit offsets?

// Matrix times one to four vectors (gemv.hip): a weighted row reduction, no MFMA.
bool gemv_applies(const GemmArgs& a, Layout layout);
int launch_gemv(const GemmArgs& a, Layout layout, hipStream_t s);

// One row per tile of gemm_kernel.hpp's menu.  `occ` = workgroups of that tile a CU can hold (LDS and
// registers), `mfma` = matrix-pipe clocks one k-slice costs one SIMD, `eff` = the measured fraction
// of the matrix-pipe rate the tile sustains with a full CU (clock-normalised), `dead` = clocks per
// slice of barrier skew and LDS latency that only other resident workgroups hide (less with the
// four-stage ring, which fetches across the barrier).
struct TileInfo { int bm, bn, bk, occ, mfma; double eff, dead; };
constexpr int kNumTiles = 8;
static const TileInfo kTiles[kNumTiles] = {
    {128, 256, 16, 2, 4096, 0.935, 350}, {128, 128, 16, 2, 2048, 0.96, 300}, {128, 64, 16, 3, 1024, 0.91, 250},
    {64, 64, 16, 5, 512, 0.88, 220},     {64, 128, 32, 2, 2048, 0.89, 478},  {64, 64, 32, 2, 1024, 0.88, 330},
    {128, 32, 32, 2, 1024, 0.85, 300},      {32, 128, 32, 2, 1024, 0.85, 300}};

struct Plan {
    int tile;          // index into kTiles
    int64_t tiles_m, tiles_n, splits, k_per_split;
    int64_t persist_grid;  // > 0: that many workgroups walk over the tiles (the kernel's tile loop); 0: one per tile
    int direct_nbw;    // > 0: the register-direct kernel (gemm_direct.hip) with blocks 16 x 16*direct_nbw ...
    int direct_ks;     // ... and the k range cut into this many parts inside a workgroup; `tile` etc. unused
};

constexpr int kCUs = 256;
constexpr int kKGran = 64;   // split-k slabs are multiples of this (a multiple of every tile's BK)

// The tiles compiled with the tile loop (gemm_kernel.hpp) and the grid it runs on: as many workgroups as
// the chip holds at once.
constexpr int kNumLoopTiles = 3;
static const int kLoopTiles[kNumLoopTiles] = {1, 2, 4};
// fraction of the matrix-pipe rate each sustains in the loop (three 128 x 64 workgroups per CU cover one
// another's tile changes better than two of the larger tiles do)
static const double kLoopEff[kNumLoopTiles] = {0.93, 0.98, 0.87};
inline int64_t loop_grid(int tile) { return (int64_t)kTiles[tile].occ * kCUs; }

// Pick (tile, k-split) with a cost model fitted to measurements on this part: when c workgroups
// share a CU, one k-slice of all of them takes  c * mfma / eff + dead / c  clocks.  Each round of
// workgroups on a CU also pays `fill`: start-up, and the output write, which is HBM-bound because
// the workgroups of a round reach their epilogues together (~9 bytes per clock per CU).  The busiest CU decides; a launch costs ~4 us of fill and drain;
// split-k adds the partial-sum traffic and a second launch.
// `tile_loop`: the product is an AB or A^T B with aligned operands, for which the tile loop is compiled.
inline Plan make_plan(int64_t M, int64_t N, int64_t K, bool b_along_k = false, int64_t conv_c = 0,
                      bool tile_loop = false) {
    const double clk = 2.4e9;
    const int64_t kslabs = cdiv(K, kKGran);
    static const int split_menu[] = {1, 2, 3, 4, 5, 6, 8, 12, 16, 24, 32};   // (5: 100 tiles x 5 fill 512 resident workgroups: 1568 x 256 x 4608 42 -> 39 us)
    Plan best{};
    double best_cost = 1e300;
    for (int ti = 0; ti < kNumTiles; ++ti) {
        const TileInfo& tl = kTiles[ti];
        const int64_t tm = cdiv(M, tl.bm), tn = cdiv(N, tl.bn);
        // the 128 x 32 tile is for tall products with few columns (a 1 x 1 convolution to a handful of
        // channels): up to four tile columns (measured ahead of the 64-wide tiles up to N = 128 on tall
        // shapes: 50176 x 96 x 1280 111 vs 139 us), so that A streams through at most four times
        if (tl.bn == 32 && tn > 4) continue;
        // ... and the 32 x 128 tile for its transpose, up to 32 rows times a large matrix: B streams through once
        if (tl.bm == 32 && tm > 1) continue;
        const double dead = tl.dead;
        // tile 0 has no k-tail handling: a k that is not a multiple of its slice depth sends every
        // tile down the register-staged path
        // ... and the 128 x 32 tile, whose few slices are all transfer issue when A comes one float at
        // a time (a convolution over 3 channels: 41 us measured against 22 us by this model)
        double slow = (ti == 0 && K % tl.bk != 0) ? 1.25 : (tl.bn == 32 && K % 4 != 0) ? 1.9 : 1.0;
        // a convolution (conv_c = its channel count) whose channels do not fill whole slices walks the
        // filter taps per lane instead of in scalar registers (8 x 224 x 224 x 16 -> 16, 3 x 3 on a
        // 32-deep tile: 68 us against 52 us by this model)
        if (conv_c > 0 && conv_c % tl.bk != 0) slow *= 1.4;
        const double fill = 3000.0 + tl.occ * tl.bm * tl.bn * 4.0 / 9.0;
        for (int sp : split_menu) {
            if (sp > 1 && kslabs < 2 * sp) break;                // keep at least 128 k per slab
            const int64_t kps = cdiv(kslabs, sp) * kKGran;
            const int64_t splits = cdiv(K, kps);
            if (splits != sp && sp > 1) continue;                // same plan as a smaller menu entry
            const int64_t wgs = tm * tn * splits;
            const double nslices = (double)cdiv(kps < K ? kps : K, tl.bk);
            const int64_t per_cu = cdiv(wgs, kCUs);              // workgroups on the busiest CU
            const int64_t full = per_cu / tl.occ, rest = per_cu % tl.occ;
            double clocks = (double)full * (nslices * (tl.occ * tl.mfma / tl.eff + dead / tl.occ) + fill);
            if (rest) clocks += nslices * (rest * tl.mfma / tl.eff + dead / rest) + fill;
            double cost = slow * clocks / clk + 4e-6;
            if (splits > 1) cost += 2.0 * splits * M * N * 4.0 / 3.0e12 + 5e-6;
            if (cost < best_cost) {
                best_cost = cost;
                best.tile = ti; best.tiles_m = tm; best.tiles_n = tn; best.splits = splits; best.k_per_split = kps;
            }
        }
    }
    // The tile loop, for short contractions with a large output: one tile per workgroup pays for the
    // multiplications and for writing C one after the other (the workgroups of a round reach their
    // epilogues together; 4096 x 4096 x 64: 17 us without its stores, 12 us for the stores alone, 28-30 us
    // together), walking over the tiles hides part of the stores under the next tile.  Fitted to
    // 4096 x 4096 x {16 ... 256}, 8192 x 8192 x 64 and others with the chip's fill of workgroups:
    // the multiplications at kLoopEff of the matrix-pipe rate plus 0.74 of the output's time at 6.7 TB/s (the
    // write-only stream rate), never less than 1.33 of the latter, plus 3.3 us.  Measured gains: K = 64
    // 30 -> 23 us, K = 128 43 -> 39, K = 256 70 -> 67, nothing from K = 512 on (and 1.5 % lost at
    // 4096^3: the hardware dispatcher balances long tiles better than a fixed stride) -- hence the cap.
    // Where it was measured ahead (0.80-0.99 of the best plain tile): at least 256 rows and 64 columns, and
    // output rows that start on cache-line boundaries.  Below 256 rows it is level or behind (64 x 100000 x 64:
    // 20.0 against 16.2 us); with a row pitch that is not a multiple of 128 bytes every tile row ends in
    // partial lines, which cost the 64-wide tile of the loop more than the 256-wide one the planner takes
    // otherwise (256 x 184280 x 48: 89 against 70 us, 8192 x 8200 x 64: 117 against 108).  The caller of this
    // function checks the pitch and base address it was given; here N stands in for a dense output.
    if (tile_loop && K <= 256 && K % 4 == 0 && N % 32 == 0 && M >= 256 && N >= 64) {
        for (int i = 0; i < kNumLoopTiles; ++i) {
            const TileInfo& tl = kTiles[kLoopTiles[i]];
            if (K < tl.bk) continue;                           // no whole slice: nothing runs ahead
            const int64_t tm = cdiv(M, tl.bm), tn = cdiv(N, tl.bn), grid = loop_grid(kLoopTiles[i]);
            if (2 * tm * tn < 3 * grid) continue;              // fewer than 1.5 tiles per workgroup: nothing to overlap
            const double mult = (double)cdiv(tm * tn, kCUs) * (double)cdiv(K, tl.bk) * tl.mfma / kLoopEff[i] / clk;
            const double write = (double)M * (double)N * 4.0 / 6.7e12;
            double cost = mult + 0.74 * write;
            if (cost < 1.33 * write) cost = 1.33 * write;
            cost += 3.3e-6;
            if (cost < best_cost) {
                best_cost = cost;
                best = Plan{};
                best.tile = kLoopTiles[i]; best.tiles_m = tm; best.tiles_n = tn; best.splits = 1;
                best.k_per_split = cdiv(K, kKGran) * kKGran;
                best.persist_grid = grid;
            }
        }
    }
    // The register-direct kernel (gemm_direct.hip): blocks of 16 x 16*nbw per wavefront, the k range
    // cut into ks parts inside a workgroup.  Fitted to launches replayed from a graph.  A wavefront
    // alone on its SIMD takes 0.05 + 0.07*nbw us per 16-deep k chunk (load latency it does not hide
    // plus the dependent MFMA chain, 0.053*nbw us of which is the matrix pipe); the register budget
    // lets 4 / 3 / 2 wavefronts (nbw = 1 / 2 / 4) share a SIMD and overlap their stalls; operands
    // come from the caches at ~15 TB/s over the whole chip (~9 TB/s once wavefronts queue behind one
    // another and contend for them) and the output costs the same; against
    // the tiled kernel's launch constant above it starts 1.1 us ahead (no staging ring to fill, no
    // barriers, a short epilogue).  Extents that rule out 16-byte accesses (K or N not a multiple
    // of 4) leave only the one-float path for A, which is worth it for a single round of small
    // blocks, or when the contraction is a few chunks deep (a filter over three channels), where the
    // tiled kernel spends its time filling and draining its ring.
    const bool one_float = (K % 4 != 0) || (N % 4 != 0);
    // A B^T (B stored N x K) with a few dozen rows against a large B: the direct blocks fetch B along k
    // in 64-byte pieces, 16 rows per access, and fall behind the tiles with k-slabs (measured:
    // 64 x 4096 x 4096 40 vs 27 us, 24 x 8192 x 8192 76 vs 49; up to 16 rows the direct blocks win)
    if (b_along_k && M > 16 && M <= 128 && K * N >= ((int64_t)1 << 22)) return best;
    for (int nbw = 1; nbw <= ((N % 4 != 0) ? 2 : 4); nbw *= 2) {
        const int occ = nbw == 1 ? 4 : nbw == 2 ? 3 : 2;
        for (int ks = 1; ks <= 4; ks *= 2) {
            const int64_t groups = cdiv(cdiv(M, 16), 4 / ks) * cdiv(N, 16 * nbw);
            if (groups > kMaxGrid) continue;
            const double waves = (double)cdiv(M, 16) * (double)cdiv(N, 16 * nbw) * ks;
            if (one_float && waves > 4 * kCUs && (K > 128 || (K > 32 && waves <= 16 * kCUs))) continue;
            if (one_float && nbw == 4 && waves <= 16 * kCUs) continue;   // measured only over many rounds
            if (one_float && ks > 1 && waves > 4 * kCUs) continue;       // k parts are for filling an idle chip
            const double chunks = (double)cdiv(cdiv(K, 16), ks);
            const double per_simd = (double)cdiv((int64_t)waves, 4 * kCUs);
            const double chain = chunks * (0.05e-6 + 0.07e-6 * nbw) * (one_float ? 1.7 : 1.0) * (double)cdiv((int64_t)per_simd, occ);
            const double pipe = per_simd * chunks * 0.053e-6 * nbw;
            const double bytes = waves * chunks * 16.0 * (16 + 16 * nbw) * 4.0 + 2.0 * M * N * 4.0;
            double cost = chain > pipe ? chain : pipe;
            const double cache_rate = waves <= 4 * kCUs ? 15e12 : 9e12;
            if (bytes / cache_rate > cost) cost = bytes / cache_rate;
            // A shallow contraction with an unaligned A over many rounds of blocks (a convolution over
            // three channels): what a block costs is its own latency chain -- row set-up, a round trip
            // for its operands, one-float loads, the stores -- spread over the wavefronts a SIMD
            // holds: measured 0.26 / 0.36 / 0.56 us per wavefront, SIMD and k chunk for nbw = 1 / 2 / 4
            // (K = 27 ... 147, 12 000 ... 100 000 blocks).
            // (measured with an aligned B and C; one float per access there too -- N not a multiple of
            // 4 -- costs 1.6 times that: 401408 x 3 x 64 50 us)
            if (one_float && waves > 16 * kCUs)
                cost = waves / (4.0 * kCUs) * (double)cdiv(K, 16) * (0.16e-6 + 0.10e-6 * nbw) * (N % 4 != 0 ? 1.6 : 1.0);
            // A B stored K x N well past the last-level cache streams from HBM in pieces as wide as the
            // block, every block of 16 rows in a pass of its own: 64-byte pieces (nbw = 1) reach about
            // 3 TB/s, wider ones 5.6-5.8 (measured: 1 x 4096 x 25088 on 16-wide blocks 133 us,
            // 16 x 8192 x 8192 on 32-wide 45 us, 1 x 16384 x 16384 on 64-wide 193 us).
            if (!b_along_k) {
                const double b_once = (double)K * (double)N * 4.0;
                if (b_once > 300e6) {
                    static const double rate[5] = {0.0, 3.0e12, 5.8e12, 0.0, 5.6e12};
                    const double hbm = b_once * (double)cdiv(M, 16) / rate[nbw];
                    if (hbm > cost) cost = hbm;
                }
            }
            cost += 6.9e-6 + (ks > 1 ? 0.3e-6 : 0.0);
            if (cost < best_cost) {
                best_cost = cost;
                best = Plan{};
                best.splits = 1;
                best.direct_nbw = nbw;
                best.direct_ks = ks;
            }
        }
    }
    return best;
}

inline size_t plan_workspace(const Plan& pl, int64_t M, int64_t N) {
    return pl.splits > 1 ? (size_t)(pl.splits * M * N) * sizeof(float) : 0;
}

// What a caller is told to bring for (M, N, K): enough for the plan of any operand layout.
inline size_t matmul_workspace(int64_t M, int64_t N, int64_t K) {
    const size_t a = plan_workspace(make_plan(M, N, K, false), M, N);
    const size_t b = plan_workspace(make_plan(M, N, K, true), M, N);
    return a > b ? a : b;
}

}  // namespace lg
