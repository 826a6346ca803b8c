// Matrix times a few vectors: C[M, N] (+)= A[M, K] B for N <= 4 (AB, and A B^T with B stored N x K).
// The paper names matrix-vector products as where its bandwidth-bound reductions come from
// (Section 4.4); with one to four output columns a matmul is exactly that:
// every element of A is used N times, so the op is a weighted row reduction bound by the read of A.
// MFMA blocks would leave 15 of 16 columns empty and, worse, fetch A in 64-byte pieces.
//
// One wavefront per row of A (per four rows when there are several columns): its lanes walk the row
// in 128-bit steps, 1 KiB contiguous per wavefront access; B comes from the caches (it is K*N floats
// for all rows); N running sums per lane and row, a butterfly over the wavefront at the end.
#include "gemm_plan.hpp"

namespace lg {

// RW rows per wavefront: with more than one column the fetches of B (N times the bytes of a row of
// A, from the caches) are shared by RW rows.
template <int NV, bool BK_CONTIG, bool VEC>
__global__ __launch_bounds__(256) void gemv_kernel(GemmArgs p) {
    constexpr int RW = NV == 1 ? 1 : 4;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t row0 = ((int64_t)blockIdx.x * 4 + wave) * RW;
    if (row0 >= p.M) return;
    const float* a[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) a[r] = p.A + (row0 + r < p.M ? row0 + r : p.M - 1) * p.lda;   // past the end: the last row again
    // B element (k, n): AB has it at B[k*ldb + n]; A B^T (and a dense single column) at B[n*bs + k]
    const int64_t bs = p.ldb;
    float acc[RW][NV];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int n = 0; n < NV; ++n) acc[r][n] = 0.f;
    // the four k of one 128-bit step: bq[e][n] = B[k + e][n]
    auto load_b = [&](int64_t k, float (&bq)[4][NV]) {
        if constexpr (BK_CONTIG) {
#pragma unroll
            for (int n = 0; n < NV; ++n) {
                const float4 b = *reinterpret_cast<const float4*>(p.B + n * bs + k);
                bq[0][n] = b.x; bq[1][n] = b.y; bq[2][n] = b.z; bq[3][n] = b.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float* b = p.B + (k + e) * bs;
                if constexpr (NV == 2) {                   // a row of B is one 8- or 16-byte load (the host checks)
                    const float2 v = *reinterpret_cast<const float2*>(b);
                    bq[e][0] = v.x; bq[e][1] = v.y;
                } else if constexpr (NV == 4) {
                    const float4 v = *reinterpret_cast<const float4*>(b);
                    bq[e][0] = v.x; bq[e][1] = v.y; bq[e][2] = v.z; bq[e][3] = v.w;
                } else {
#pragma unroll
                    for (int n = 0; n < NV; ++n) bq[e][n] = b[n];
                }
            }
        }
    };
    auto step = [&](int64_t j) {                               // 128-bit step j of every row of the wavefront
        float bq[4][NV];
        float4 v[RW];
#pragma unroll
        for (int r = 0; r < RW; ++r) v[r] = *reinterpret_cast<const float4*>(a[r] + 4 * j);
        load_b(4 * j, bq);
#pragma unroll
        for (int r = 0; r < RW; ++r)
#pragma unroll
            for (int n = 0; n < NV; ++n)
                acc[r][n] += (v[r].x * bq[0][n] + v[r].y * bq[1][n]) + (v[r].z * bq[2][n] + v[r].w * bq[3][n]);
    };
    if constexpr (VEC) {
        const int64_t n4 = p.K / 4;
        int64_t j = lane;
        constexpr int U = RW == 1 ? 4 : 1;                     // steps in flight per lane (RW rows each)
        for (; j + (U - 1) * kWave < n4; j += U * kWave) {
#pragma unroll
            for (int u = 0; u < U; ++u) step(j + u * kWave);
        }
        for (; j < n4; j += kWave) step(j);
    } else {
        for (int64_t k = lane; k < p.K; k += kWave) {
#pragma unroll
            for (int n = 0; n < NV; ++n) {
                const float b = BK_CONTIG ? p.B[n * bs + k] : p.B[k * bs + n];
#pragma unroll
                for (int r = 0; r < RW; ++r) acc[r][n] += a[r][k] * b;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int n = 0; n < NV; ++n) {
            const float s = wave_sum(acc[r][n]);
            if (lane == 0 && row0 + r < p.M) {
                float* c = p.C + (row0 + r) * p.ldc + n;
                *c = p.accumulate ? *c + s : s;
            }
        }
}

// Worth it when the rows are long enough to keep a wavefront busy and there are enough of them to
// fill the chip (otherwise the register-direct kernel's k parts do better), and when B can be
// fetched in whole rows or along k: A B^T; AB with one column, or with two or four columns whose
// rows are 8- / 16-byte aligned.
bool gemv_applies(const GemmArgs& a, Layout layout) {
    if (a.N < 1 || a.N > 4 || a.K < 1024 || a.M < 1024) return false;
    if (layout == Layout::NT) return true;
    if (layout != Layout::NN) return false;
    if (a.N == 1) return true;
    const uintptr_t b = reinterpret_cast<uintptr_t>(a.B);
    if (a.N == 2) return a.ldb % 2 == 0 && b % 8 == 0;
    if (a.N == 4) return a.ldb % 4 == 0 && b % 16 == 0;
    return false;
}

int launch_gemv(const GemmArgs& a, Layout layout, hipStream_t s) {
    if (!gemv_applies(a, layout)) return LG_ERR_UNSUPPORTED;
    const int64_t blocks = cdiv(a.M, 4 * (a.N == 1 ? 1 : 4));          // 4 wavefronts x RW rows
    if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
    // a dense single column of AB is contiguous along k like the rows of B in A B^T
    const bool bk = layout == Layout::NT || (a.N == 1 && a.ldb == 1);
    const bool vec = a.K % 4 == 0 && a.lda % 4 == 0 && aligned16(a.A) &&
                     (!bk || ((a.ldb % 4 == 0 || a.N == 1) && aligned16(a.B)));
    const dim3 g((unsigned)blocks), b(256);
#define LG_GEMV(NV)                                                                                   \
    do {                                                                                              \
        if (bk && vec)  hipLaunchKernelGGL((gemv_kernel<NV, true, true>), g, b, 0, s, a);             \
        else if (bk)    hipLaunchKernelGGL((gemv_kernel<NV, true, false>), g, b, 0, s, a);            \
        else if (vec)   hipLaunchKernelGGL((gemv_kernel<NV, false, true>), g, b, 0, s, a);            \
        else            hipLaunchKernelGGL((gemv_kernel<NV, false, false>), g, b, 0, s, a);           \
    } while (0)
    switch (a.N) {
        case 1: LG_GEMV(1); break;
        case 2: LG_GEMV(2); break;
        case 3: LG_GEMV(3); break;
        default: LG_GEMV(4); break;
    }
#undef LG_GEMV
    return launch_status();
}

}  // namespace lg
