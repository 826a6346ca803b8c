// Matmul (Section 4.6.1: AB, A^T B, A B^T) and conv_2d_nhwc_hwcf (Section 4.6.2): host side of the
// MFMA GEMM kernel in gemm_kernel.hpp -- argument checks, plan, launch, split-k combine.
#include "gemm_kernel.hpp"

namespace lg {

void launch_nn(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s) { launch_planned<false, false, false>(a, pl, vec, s); }
void launch_conv(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s) { launch_planned<true, false, false>(a, pl, vec, s); }

// out[m,n] (+)= sum_z partial[z][m,n]; slabs are dense M x N.  Fixed order: z ascending.
__global__ __launch_bounds__(256) void splitk_combine_kernel(
    const float* __restrict__ partial, float* __restrict__ C,
    int64_t M, int64_t N, int64_t ldc, int splits, int accumulate) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * N) return;
    const int64_t m = idx / N, n = idx - m * N;
    float s = 0.f;
    for (int z = 0; z < splits; ++z) s += partial[(int64_t)z * M * N + idx];
    float* cp = C + m * ldc + n;
    *cp = accumulate ? *cp + s : s;
}

__global__ __launch_bounds__(256) void fill_zero_2d_kernel(float* C, int64_t M, int64_t N, int64_t ldc) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * N) return;
    const int64_t m = idx / N;
    C[m * ldc + (idx - m * N)] = 0.f;
}

enum class Layout { NN, CONV, TN, NT };

static int run_gemm(GemmArgs a, Layout layout, bool vec, int user_accumulate, void* workspace,
                    size_t workspace_bytes, hipStream_t s) {
    const Plan pl = make_plan(a.M, a.N, a.K);
    const size_t need = plan_workspace(pl, a.M, a.N);
    if (need > 0) {
        if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
            return LG_ERR_WORKSPACE;
    }
    if (pl.tiles_m * pl.tiles_n > kMaxGrid || pl.splits > 65535) return LG_ERR_UNSUPPORTED;
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
        const int64_t blocks = cdiv(a.M * a.N, 256);
        if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(splitk_combine_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                           static_cast<const float*>(workspace), Cfinal, a.M, a.N, ldc_final, (int)pl.splits,
                           user_accumulate);
        return launch_status();
    }
    return LG_OK;
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
    const Plan pl = make_plan(M, N, K);
    if (block_m) *block_m = kTiles[pl.tile].bm;
    if (block_n) *block_n = kTiles[pl.tile].bn;
    if (k_splits) *k_splits = (int)pl.splits;
    return LG_OK;
}

extern "C" size_t lg_matmul_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    using namespace lg;
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return plan_workspace(make_plan(M, N, K), M, N);
}

extern "C" int lg_matmul(const float* A, const float* B, float* C,
                         int64_t M, int64_t N, int64_t K,
                         int64_t lda, int64_t ldb, int64_t ldc,
                         int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace lg;
    if (M < 0 || N < 0 || K < 0 || lda < K || ldb < N || ldc < N) return LG_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return LG_OK;
    if (!C || (K > 0 && (!A || !B))) return LG_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t c_bytes = ((M - 1) * ldc + N) * 4;
    if (K == 0) return accumulate ? LG_OK : zero_output(C, M, N, ldc, s);
    if (overlaps(A, ((M - 1) * lda + K) * 4, C, c_bytes) || overlaps(B, ((K - 1) * ldb + N) * 4, C, c_bytes))
        return LG_ERR_INVALID_ARG;
    if (M >= (int64_t)1 << 31 || N >= (int64_t)1 << 31 || K >= (int64_t)1 << 31) return LG_ERR_UNSUPPORTED;
    const bool vec = (K % 4 == 0) && (N % 4 == 0) && (lda % 4 == 0) && (ldb % 4 == 0) && (ldc % 4 == 0) &&
                     aligned16(A) && aligned16(B) && aligned16(C);
    GemmArgs a{};
    a.A = A; a.B = B; a.C = C;
    a.M = M; a.N = N; a.K = K;
    a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    return run_gemm(a, Layout::NN, vec, accumulate, workspace, workspace_bytes, s);
}

extern "C" int lg_matmul_t(const float* A, const float* B, float* C,
                           int64_t M, int64_t N, int64_t K,
                           int64_t lda, int64_t ldb, int64_t ldc,
                           int transA, int transB,
                           int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace lg;
    if (!transA && !transB)
        return lg_matmul(A, B, C, M, N, K, lda, ldb, ldc, accumulate, workspace, workspace_bytes, stream);
    if (M < 0 || N < 0 || K < 0 || ldc < N) return LG_ERR_INVALID_ARG;
    const int64_t a_rows = transA ? K : M, a_cols = transA ? M : K;     // stored shape of A
    const int64_t b_rows = transB ? N : K, b_cols = transB ? K : N;     // stored shape of B
    if (lda < a_cols || ldb < b_cols) return LG_ERR_INVALID_ARG;
    if (transA && transB) return LG_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return LG_OK;
    if (!C || (K > 0 && (!A || !B))) return LG_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t c_bytes = ((M - 1) * ldc + N) * 4;
    if (K == 0) return accumulate ? LG_OK : zero_output(C, M, N, ldc, s);
    if (overlaps(A, ((a_rows - 1) * lda + a_cols) * 4, C, c_bytes) ||
        overlaps(B, ((b_rows - 1) * ldb + b_cols) * 4, C, c_bytes))
        return LG_ERR_INVALID_ARG;
    if (M >= (int64_t)1 << 31 || N >= (int64_t)1 << 31 || K >= (int64_t)1 << 31) return LG_ERR_UNSUPPORTED;
    const bool vec = (K % 4 == 0) && (N % 4 == 0) && (M % 4 == 0 || !transA) && (lda % 4 == 0) && (ldb % 4 == 0) &&
                     (ldc % 4 == 0) && aligned16(A) && aligned16(B) && aligned16(C);
    GemmArgs a{};
    a.A = A; a.B = B; a.C = C;
    a.M = M; a.N = N; a.K = K;
    a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    return run_gemm(a, transA ? Layout::TN : Layout::NT, vec, accumulate, workspace, workspace_bytes, s);
}

extern "C" size_t lg_conv2d_workspace_bytes(int64_t N, int64_t H, int64_t W, int64_t C,
                                            int64_t KH, int64_t KW, int64_t F,
                                            int64_t SH, int64_t SW, int64_t DH, int64_t DW) {
    using namespace lg;
    const int64_t OH = lg_conv_out_extent(H, KH, SH, DH), OW = lg_conv_out_extent(W, KW, SW, DW);
    if (N <= 0 || C <= 0 || F <= 0 || OH <= 0 || OW <= 0) return 0;
    const int64_t M = N * OH * OW;
    return plan_workspace(make_plan(M, F, KH * KW * C), M, F);
}

extern "C" int lg_conv2d_nhwc_hwcf(const float* I, const float* Kf, float* O,
                                   int64_t N, int64_t H, int64_t W, int64_t C,
                                   int64_t KH, int64_t KW, int64_t F,
                                   int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                                   int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace lg;
    if (N < 0 || H < 0 || W < 0 || C < 0 || KH < 1 || KW < 1 || F < 0) return LG_ERR_INVALID_ARG;
    if (SH < 1 || SW < 1 || DH < 1 || DW < 1) return LG_ERR_INVALID_ARG;
    if (N == 0 || F == 0) return LG_OK;
    const int64_t OH = lg_conv_out_extent(H, KH, SH, DH), OW = lg_conv_out_extent(W, KW, SW, DW);
    if (OH == 0 || OW == 0) return LG_ERR_INVALID_ARG;
    if (!O || (C > 0 && (!I || !Kf))) return LG_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
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
        return run_gemm(mm, Layout::NN, vec, accumulate, workspace, workspace_bytes, s);
    }
    GemmArgs a{};
    a.A = I; a.B = Kf; a.C = O;
    a.M = M; a.N = F; a.K = Kg;
    a.lda = 0; a.ldb = F; a.ldc = F;
    a.g = ConvGeom{H, W, C, KW, SH, SW, DH, DW, OH, OW};
    return run_gemm(a, Layout::CONV, vec, accumulate, workspace, workspace_bytes, s);
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
