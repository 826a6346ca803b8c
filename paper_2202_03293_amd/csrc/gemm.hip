// Matmul (Section 4.6.1: AB, A^T B, A B^T) and conv_2d_nhwc_hwcf (Section 4.6.2): host side of the
// MFMA GEMM kernel in gemm_kernel.hpp -- argument checks, plan, launch, split-k combine.
#include "gemm_kernel.hpp"

namespace lg {

void launch_nn(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s) { launch_planned<false, false, false>(a, pl, vec, s); }
void launch_conv(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s) { launch_planned<true, false, false>(a, pl, vec, s); }

// out[m,n] (+)= sum_z partial[z][m,n]; slabs are dense M x N.  Fixed order: z ascending, eight slabs
// at a time, all eight requested before the first add (the kernel is memory round trips long: one per
// eight slabs instead of one per slab).  V = 4: four adjacent columns per lane, 128-bit accesses
// (N and ldc multiples of 4, C 16-byte aligned); V = 1 otherwise.
template <int V>
__global__ __launch_bounds__(256) void splitk_combine_kernel(
    const float* __restrict__ partial, float* __restrict__ C,
    int64_t M, int64_t N, int64_t ldc, int splits, int accumulate) {
    const int64_t idx = ((int64_t)blockIdx.x * 256 + threadIdx.x) * V;
    if (idx >= M * N) return;
    const int64_t m = idx / N, n = idx - m * N;
    float s[V];
#pragma unroll
    for (int e = 0; e < V; ++e) s[e] = 0.f;
    for (int z0 = 0; z0 < splits; z0 += 8) {
        float v[8][V];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float* q = partial + (int64_t)(z0 + u < splits ? z0 + u : z0) * M * N + idx;
            if constexpr (V == 4) {
                const float4 t = *reinterpret_cast<const float4*>(q);
                v[u][0] = t.x; v[u][1] = t.y; v[u][2] = t.z; v[u][3] = t.w;
            } else {
                v[u][0] = *q;
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (z0 + u < splits) {
#pragma unroll
                for (int e = 0; e < V; ++e) s[e] += v[u][e];
            }
    }
    float* cp = C + m * ldc + n;
    if constexpr (V == 4) {
        float4 o = make_float4(s[0], s[1], s[2], s[3]);
        if (accumulate) {
            const float4 c = *reinterpret_cast<const float4*>(cp);
            o.x += c.x; o.y += c.y; o.z += c.z; o.w += c.w;
        }
        *reinterpret_cast<float4*>(cp) = o;
    } else {
        *cp = accumulate ? *cp + s[0] : s[0];
    }
}

__global__ __launch_bounds__(256) void fill_zero_2d_kernel(float* C, int64_t M, int64_t N, int64_t ldc) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * N) return;
    const int64_t m = idx / N;
    C[m * ldc + (idx - m * N)] = 0.f;
}

// The menu a caller may pick from by number: the eight tiles, then the register-direct kernel with
// blocks 16 x {16, 32, 64} and {1, 2, 4} k parts per workgroup, then the tiles that have a tile loop,
// run with it (where the loop is not compiled -- A B^T, convolutions, unaligned operands -- or there are no
// more tiles than workgroups, they run as the plain tile).
constexpr int kNumDirect = 9;
constexpr int kNumVariants = kNumTiles + kNumDirect + kNumLoopTiles;

// The plan of a forced variant; false when the numbers make no sense.
static bool forced_plan(int64_t M, int64_t N, int64_t K, int variant, int k_splits, Plan* out) {
    if (variant < 0 || variant >= kNumVariants || k_splits < 1 || k_splits > 65535) return false;
    Plan pl{};
    if (variant >= kNumTiles + kNumDirect) {
        if (k_splits != 1) return false;
        const int tile = kLoopTiles[variant - kNumTiles - kNumDirect];
        if (!forced_plan(M, N, K, tile, 1, &pl)) return false;
        // the chip's fill of workgroups, or a third of the tiles if that is fewer (so that small shapes loop too)
        const int64_t third = pl.tiles_m * pl.tiles_n / 3 / kXcds * kXcds;
        pl.persist_grid = third < kXcds ? kXcds : third < loop_grid(tile) ? third : loop_grid(tile);
    } else if (variant >= kNumTiles) {
        static const int pow2[3] = {1, 2, 4};
        if (k_splits != 1) return false;
        pl.direct_nbw = pow2[(variant - kNumTiles) / 3];
        pl.direct_ks = pow2[(variant - kNumTiles) % 3];
        pl.splits = 1;
    } else {
        const TileInfo& tl = kTiles[variant];
        pl.tile = variant;
        pl.tiles_m = cdiv(M, tl.bm);
        pl.tiles_n = cdiv(N, tl.bn);
        pl.k_per_split = cdiv(cdiv(K, kKGran), k_splits) * kKGran;
        pl.splits = cdiv(K, pl.k_per_split);       // <= k_splits: slabs are whole multiples of the granule
    }
    *out = pl;
    return true;
}

// bytes from an operand's base to the end of its last element, as stored
static int64_t operand_bytes_a(const GemmArgs& a, Layout layout) {
    if (layout == Layout::CONV) {                  // dense NHWC input: batch = M / (OH * OW)
        const int64_t n = a.M / (a.g.OH * a.g.OW);
        return n * a.g.H * a.g.W * a.g.C * 4;
    }
    const int64_t rows = layout == Layout::TN ? a.K : a.M, cols = layout == Layout::TN ? a.M : a.K;
    return ((rows - 1) * a.lda + cols) * 4;
}
static int64_t operand_bytes_b(const GemmArgs& a, Layout layout) {
    const int64_t rows = layout == Layout::NT ? a.N : a.K, cols = layout == Layout::NT ? a.K : a.N;
    return ((rows - 1) * a.ldb + cols) * 4;
}

static int run_plan(GemmArgs a, Layout layout, bool vec, const Plan& pl, int user_accumulate, void* workspace,
                    size_t workspace_bytes, hipStream_t s) {
    if (pl.direct_nbw > 0) {
        a.accumulate = user_accumulate;
        return launch_direct(a, layout, pl.direct_nbw, pl.direct_ks, s);
    }
    const size_t need = plan_workspace(pl, a.M, a.N);
    if (need > 0) {
        if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
            return LG_ERR_WORKSPACE;
        // partial sums written over an operand or the output would give wrong numbers, not an error
        if (overlaps(workspace, (int64_t)need, a.C, ((a.M - 1) * a.ldc + a.N) * 4) ||
            overlaps(workspace, (int64_t)need, a.A, operand_bytes_a(a, layout)) ||
            overlaps(workspace, (int64_t)need, a.B, operand_bytes_b(a, layout)))
            return LG_ERR_INVALID_ARG;
    }
    // every launch of the call is checked against the grid limits before the first one is enqueued
    if (pl.tiles_m * pl.tiles_n > kMaxGrid || pl.splits > 65535) return LG_ERR_UNSUPPORTED;
    if (pl.splits > 1 && cdiv(a.M * a.N, 256) > kMaxGrid) return LG_ERR_UNSUPPORTED;
    float* Cfinal = a.C;
    const int64_t ldc_final = a.ldc;
    a.tiles_m = (unsigned)pl.tiles_m;
    a.tiles_n = (unsigned)pl.tiles_n;
    a.k_per_split = pl.k_per_split;
    if (pl.splits > 1) {
        a.C = static_cast<float*>(workspace);
        a.ldc = a.N;
        a.accumulate = 0;
    } else {
        a.accumulate = user_accumulate;
    }
    switch (layout) {
        case Layout::NN: launch_nn(a, pl, vec, s); break;
        case Layout::CONV: launch_conv(a, pl, vec, s); break;
        case Layout::TN: launch_tn(a, pl, vec, s); break;
        case Layout::NT: launch_nt(a, pl, vec, s); break;
    }
    if (launch_status() != LG_OK) return LG_ERR_RUNTIME;
    if (pl.splits > 1) {
        // (the workspace is 256-byte aligned and its slabs are M*N floats: whole quads when N is a multiple of 4)
        if (a.N % 4 == 0 && ldc_final % 4 == 0 && aligned16(Cfinal))
            hipLaunchKernelGGL(splitk_combine_kernel<4>, dim3((unsigned)cdiv(a.M * a.N / 4, 256)), dim3(256), 0, s,
                               static_cast<const float*>(workspace), Cfinal, a.M, a.N, ldc_final, (int)pl.splits,
                               user_accumulate);
        else
            hipLaunchKernelGGL(splitk_combine_kernel<1>, dim3((unsigned)cdiv(a.M * a.N, 256)), dim3(256), 0, s,
                               static_cast<const float*>(workspace), Cfinal, a.M, a.N, ldc_final, (int)pl.splits,
                               user_accumulate);
        return launch_status();
    }
    return LG_OK;
}

// variant < 0: the planner decides
static int run_gemm(const GemmArgs& a, Layout layout, bool vec, int user_accumulate, void* workspace,
                    size_t workspace_bytes, hipStream_t s, int variant = -1, int k_splits = 1) {
    Plan pl{};
    if (variant < 0) {
        if (gemv_applies(a, layout)) {
            GemmArgs g = a;
            g.accumulate = user_accumulate;
            return launch_gemv(g, layout, s);
        }
        pl = make_plan(a.M, a.N, a.K, layout == Layout::NT, layout == Layout::CONV ? a.g.C : 0,
                       // (an accumulating epilogue waits for C: nothing to hide, 57 vs 49 us at 4096 x 4096 x 64;
                       // output rows off the cache-line grid: see make_plan)
                       (layout == Layout::NN || layout == Layout::TN) && vec && !user_accumulate &&
                           a.ldc % 32 == 0 && (reinterpret_cast<uintptr_t>(a.C) & 127u) == 0);
        // the planner knows extents, not pitches: operands padded past the direct kernel's reach
        // run on the smallest tile, unsplit (which needs no workspace either)
        if (pl.direct_nbw > 0 && !direct_can_run(a, layout)) forced_plan(a.M, a.N, a.K, 3, 1, &pl);
        // Operands that turn out unaligned (the planner saw only extents): one float per load costs
        // the wider blocks more registers than they have, and more than one round of small blocks
        // is the tiled kernel's business.
        if (pl.direct_nbw > 0 && !vec && a.K % 4 == 0 && a.N % 4 == 0) {
            if (cdiv(a.M, 16) * cdiv(a.N, 16) * pl.direct_ks > 4 * kCUs) forced_plan(a.M, a.N, a.K, 3, 1, &pl);
            else pl.direct_nbw = 1;
        }
    } else if (!forced_plan(a.M, a.N, a.K, variant, k_splits, &pl)) {
        return LG_ERR_INVALID_ARG;
    }
    return run_plan(a, layout, vec, pl, user_accumulate, workspace, workspace_bytes, s);
}

static int zero_output(float* C, int64_t M, int64_t N, int64_t ldc, hipStream_t s) {
    const int64_t blocks = cdiv(M * N, 256);
    if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(fill_zero_2d_kernel, dim3((unsigned)blocks), dim3(256), 0, s, C, M, N, ldc);
    return launch_status();
}

}  // namespace lg

extern "C" int lg_matmul_plan(int64_t M, int64_t N, int64_t K, int* block_m, int* block_n, int* k_splits) {
    using namespace lg;
    if (M <= 0 || N <= 0 || K <= 0) return LG_ERR_INVALID_ARG;
    const Plan pl = make_plan(M, N, K, false, 0, true);
    const bool direct = pl.direct_nbw > 0;
    if (block_m) *block_m = direct ? 16 : kTiles[pl.tile].bm;
    if (block_n) *block_n = direct ? 16 * pl.direct_nbw : kTiles[pl.tile].bn;
    if (k_splits) *k_splits = direct ? 1 : (int)pl.splits;
    return LG_OK;
}

extern "C" int lg_matmul_plan_tile_loop(int64_t M, int64_t N, int64_t K) {
    using namespace lg;
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return make_plan(M, N, K, false, 0, true).persist_grid > 0;
}

extern "C" size_t lg_matmul_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    using namespace lg;
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return matmul_workspace(M, N, K);
}

extern "C" int lg_matmul_t_plan(int64_t M, int64_t N, int64_t K, int transA, int transB,
                                int* block_m, int* block_n, int* k_splits) {
    using namespace lg;
    if (M <= 0 || N <= 0 || K <= 0 || (transA && transB)) return LG_ERR_INVALID_ARG;
    const Plan pl = make_plan(M, N, K, transB != 0, 0, !transB);
    const bool direct = pl.direct_nbw > 0;
    if (block_m) *block_m = direct ? 16 : kTiles[pl.tile].bm;
    if (block_n) *block_n = direct ? 16 * pl.direct_nbw : kTiles[pl.tile].bn;
    if (k_splits) *k_splits = direct ? 1 : (int)pl.splits;
    return LG_OK;
}

namespace lg {

// C (+)= op(A) op(B) in any of the three layouts; variant < 0 leaves the choice of kernel to the planner.
static int matmul_impl(const float* A, const float* B, float* C, int64_t M, int64_t N, int64_t K,
                       int64_t lda, int64_t ldb, int64_t ldc, int transA, int transB, int accumulate,
                       void* workspace, size_t workspace_bytes, void* stream, int variant, int k_splits) {
    if (M < 0 || N < 0 || K < 0 || ldc < N) return LG_ERR_INVALID_ARG;
    const int64_t a_rows = transA ? K : M, a_cols = transA ? M : K;     // stored shape of A
    const int64_t b_rows = transB ? N : K, b_cols = transB ? K : N;     // stored shape of B
    if (lda < a_cols || ldb < b_cols) return LG_ERR_INVALID_ARG;
    if (transA && transB) return LG_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return LG_OK;
    if (!C || (K > 0 && (!A || !B))) return LG_ERR_INVALID_ARG;
    hipStream_t s = begin_call(stream);
    const int64_t c_bytes = ((M - 1) * ldc + N) * 4;
    if (K == 0) return accumulate ? LG_OK : zero_output(C, M, N, ldc, s);
    if (overlaps(A, ((a_rows - 1) * lda + a_cols) * 4, C, c_bytes) ||
        overlaps(B, ((b_rows - 1) * ldb + b_cols) * 4, C, c_bytes))
        return LG_ERR_INVALID_ARG;
    if (M >= (int64_t)1 << 31 || N >= (int64_t)1 << 31 || K >= (int64_t)1 << 31) return LG_ERR_UNSUPPORTED;
    // 128-bit transfers need every operand row to start on a 16-byte boundary and hold whole quads.
    // A B^T fetches both operands along k and writes C one float per lane in dense rows, so there
    // the output (N, ldc, C's base) does not enter into it: a product against a [vocabulary x hidden]
    // matrix with an odd vocabulary keeps its 128-bit loads.
    const bool vec = transB ? (K % 4 == 0) && (lda % 4 == 0) && (ldb % 4 == 0) && aligned16(A) && aligned16(B)
                            : (K % 4 == 0) && (N % 4 == 0) && (M % 4 == 0 || !transA) && (lda % 4 == 0) &&
                              (ldb % 4 == 0) && (ldc % 4 == 0) && aligned16(A) && aligned16(B) && aligned16(C);
    GemmArgs a{};
    a.A = A; a.B = B; a.C = C;
    a.M = M; a.N = N; a.K = K;
    a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    const Layout layout = transA ? Layout::TN : transB ? Layout::NT : Layout::NN;
    return run_gemm(a, layout, vec, accumulate, workspace, workspace_bytes, s, variant, k_splits);
}

}  // namespace lg

extern "C" int lg_matmul(const float* A, const float* B, float* C,
                         int64_t M, int64_t N, int64_t K,
                         int64_t lda, int64_t ldb, int64_t ldc,
                         int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    return lg::matmul_impl(A, B, C, M, N, K, lda, ldb, ldc, 0, 0, accumulate, workspace, workspace_bytes, stream, -1, 1);
}

extern "C" int lg_matmul_t(const float* A, const float* B, float* C,
                           int64_t M, int64_t N, int64_t K,
                           int64_t lda, int64_t ldb, int64_t ldc,
                           int transA, int transB,
                           int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    return lg::matmul_impl(A, B, C, M, N, K, lda, ldb, ldc, transA, transB, accumulate, workspace, workspace_bytes,
                           stream, -1, 1);
}

extern "C" int lg_gemm_variants(void) { return lg::kNumVariants; }

extern "C" int lg_gemm_variant_info(int variant, int* block_m, int* block_n, int* block_k, int* k_parts,
                                    int* tile_loop) {
    using namespace lg;
    Plan pl{};
    if (!forced_plan(1, 1, 1, variant, 1, &pl)) return LG_ERR_INVALID_ARG;
    const bool direct = pl.direct_nbw > 0;
    if (block_m) *block_m = direct ? 16 : kTiles[pl.tile].bm;
    if (block_n) *block_n = direct ? 16 * pl.direct_nbw : kTiles[pl.tile].bn;
    if (block_k) *block_k = direct ? 16 : kTiles[pl.tile].bk;
    if (k_parts) *k_parts = direct ? pl.direct_ks : 1;
    if (tile_loop) *tile_loop = pl.persist_grid > 0;
    return LG_OK;
}

extern "C" size_t lg_gemm_variant_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant, int k_splits) {
    using namespace lg;
    Plan pl{};
    if (M <= 0 || N <= 0 || K <= 0 || !forced_plan(M, N, K, variant, k_splits, &pl)) return 0;
    return pl.direct_nbw > 0 ? 0 : plan_workspace(pl, M, N);
}

extern "C" int lg_matmul_variant(const float* A, const float* B, float* C,
                                 int64_t M, int64_t N, int64_t K,
                                 int64_t lda, int64_t ldb, int64_t ldc,
                                 int transA, int transB, int accumulate,
                                 int variant, int k_splits,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    if (variant < 0) return LG_ERR_INVALID_ARG;
    return lg::matmul_impl(A, B, C, M, N, K, lda, ldb, ldc, transA, transB, accumulate, workspace, workspace_bytes,
                           stream, variant, k_splits);
}

extern "C" size_t lg_conv2d_workspace_bytes(int64_t N, int64_t H, int64_t W, int64_t C,
                                            int64_t KH, int64_t KW, int64_t F,
                                            int64_t SH, int64_t SW, int64_t DH, int64_t DW) {
    using namespace lg;
    const int64_t OH = lg_conv_out_extent(H, KH, SH, DH), OW = lg_conv_out_extent(W, KW, SW, DW);
    if (N <= 0 || C <= 0 || F <= 0 || OH <= 0 || OW <= 0) return 0;
    const int64_t M = N * OH * OW;
    // the plan lg_conv2d_nhwc_hwcf will make: a 1 x 1 filter at stride 1 runs as the matmul it is
    const bool as_matmul = KH == 1 && KW == 1 && SH == 1 && SW == 1;
    return plan_workspace(make_plan(M, F, KH * KW * C, false, as_matmul ? 0 : C), M, F);
}

namespace lg {

static int conv2d_impl(const float* I, const float* Kf, float* O,
                       int64_t N, int64_t H, int64_t W, int64_t C,
                       int64_t KH, int64_t KW, int64_t F,
                       int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                       int accumulate, void* workspace, size_t workspace_bytes, void* stream,
                       int variant, int k_splits) {
    if (N < 0 || H < 0 || W < 0 || C < 0 || KH < 1 || KW < 1 || F < 0) return LG_ERR_INVALID_ARG;
    if (SH < 1 || SW < 1 || DH < 1 || DW < 1) return LG_ERR_INVALID_ARG;
    if (N == 0 || F == 0) return LG_OK;
    const int64_t OH = lg_conv_out_extent(H, KH, SH, DH), OW = lg_conv_out_extent(W, KW, SW, DW);
    if (OH == 0 || OW == 0) return LG_ERR_INVALID_ARG;
    if (!O || (C > 0 && (!I || !Kf))) return LG_ERR_INVALID_ARG;
    hipStream_t s = begin_call(stream);
    const int64_t M = N * OH * OW, Kg = KH * KW * C;
    if (Kg == 0) return accumulate ? LG_OK : zero_output(O, M, F, F, s);
    if (overlaps(I, N * H * W * C * 4, O, M * F * 4) || overlaps(Kf, Kg * F * 4, O, M * F * 4))
        return LG_ERR_INVALID_ARG;
    if (M >= (int64_t)1 << 31 || F >= (int64_t)1 << 31 || Kg >= (int64_t)1 << 31) return LG_ERR_UNSUPPORTED;
    const bool vec = (C % 4 == 0) && (F % 4 == 0) && aligned16(I) && aligned16(Kf) && aligned16(O);
    if (KH == 1 && KW == 1 && SH == 1 && SW == 1) {
        // a 1x1 filter at stride 1 reads every pixel once: the input already is the row-major M x C matrix
        GemmArgs mm{};
        mm.A = I; mm.B = Kf; mm.C = O;
        mm.M = M; mm.N = F; mm.K = C;
        mm.lda = C; mm.ldb = F; mm.ldc = F;
        return run_gemm(mm, Layout::NN, vec, accumulate, workspace, workspace_bytes, s, variant, k_splits);
    }
    GemmArgs a{};
    a.A = I; a.B = Kf; a.C = O;
    a.M = M; a.N = F; a.K = Kg;
    a.lda = 0; a.ldb = F; a.ldc = F;
    a.g = ConvGeom{H, W, C, KW, SH, SW, DH, DW, OH, OW};
    return run_gemm(a, Layout::CONV, vec, accumulate, workspace, workspace_bytes, s, variant, k_splits);
}

}  // namespace lg

extern "C" int lg_conv2d_nhwc_hwcf(const float* I, const float* Kf, float* O,
                                   int64_t N, int64_t H, int64_t W, int64_t C,
                                   int64_t KH, int64_t KW, int64_t F,
                                   int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                                   int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    return lg::conv2d_impl(I, Kf, O, N, H, W, C, KH, KW, F, SH, SW, DH, DW, accumulate, workspace, workspace_bytes,
                           stream, -1, 1);
}

extern "C" int lg_conv2d_nhwc_hwcf_variant(const float* I, const float* Kf, float* O,
                                           int64_t N, int64_t H, int64_t W, int64_t C,
                                           int64_t KH, int64_t KW, int64_t F,
                                           int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                                           int accumulate, int variant, int k_splits,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    if (variant < 0) return LG_ERR_INVALID_ARG;
    return lg::conv2d_impl(I, Kf, O, N, H, W, C, KH, KW, F, SH, SW, DH, DW, accumulate, workspace, workspace_bytes,
                           stream, variant, k_splits);
}

extern "C" size_t lg_conv1d_workspace_bytes(int64_t N, int64_t W, int64_t C, int64_t KW, int64_t F,
                                            int64_t SW, int64_t DW) {
    return lg_conv2d_workspace_bytes(N, 1, W, C, 1, KW, F, 1, SW, 1, DW);
}

extern "C" int lg_conv1d_nwc_wcf(const float* I, const float* Kf, float* O,
                                 int64_t N, int64_t W, int64_t C, int64_t KW, int64_t F,
                                 int64_t SW, int64_t DW,
                                 int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    return lg_conv2d_nhwc_hwcf(I, Kf, O, N, 1, W, C, 1, KW, F, 1, SW, 1, DW, accumulate, workspace,
                               workspace_bytes, stream);
}
