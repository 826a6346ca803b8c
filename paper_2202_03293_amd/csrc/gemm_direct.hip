// Small and skinny GEMMs: the same operations as gemm_kernel.hpp (Section 4.6.1 matmuls in their
// three layouts, Section 4.6.2 convolution as an implicit GEMM), for problems on which the tiled
// kernel leaves most of the chip idle or waits on its own staging: a handful of output tiles, or a
// contraction only a few k-slices deep (a first-layer convolution: K = KH*KW*3).
//
// No LDS staging and no barriers in the k loop: each wavefront owns a 16 x (16*NBW) block of C and
// loads its operands from global memory straight into the register layout of
// v_mfma_f32_16x16x4_f32, several 16-deep k chunks ahead of the multiply.  A workgroup is four such
// wavefronts: four row blocks (ks = 1), or fewer row blocks whose k range is cut into ks parts that
// are summed through LDS at the end, in ascending order of k.  Small blocks mean many wavefronts
// (a 256 x 256 problem gives 256 of them instead of 16 tiles of 64 x 64) and a short dependent
// chain per wavefront, which is what a launch-bound problem needs; operands are re-read from the
// caches more often than with LDS tiles, which is why large problems stay on the tiled kernel.
//
// k order inside a chunk: lane group g = lane / 16 of MFMA step j multiplies k = chunk + 4g + j,
// for both operands (the sum over k is order-free), so a lane whose operand is contiguous along k
// fetches its four values of a chunk with one 16-byte load.
#include "gemm_kernel.hpp"

namespace lg {

typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int NBW>
struct DirectFrag {
    float a[4];            // A[row][chunk + 4g + j]
    float b[NBW][4];       // B[chunk + 4g + j][column of block nb]
};

// LAYOUT: 0 = AB, 1 = convolution, 2 = A^T B, 3 = A B^T.  a_vec / b_vec: the operand that is
// contiguous along k may be fetched 16 bytes at a time (row pitch and base 16-byte aligned).
template <int LAYOUT, int NBW>
__global__ __launch_bounds__(256) void gemm_direct_kernel(GemmArgs p, int ks, int a_vec, int b_vec) {
    constexpr bool CONV = LAYOUT == 1, TA = LAYOUT == 2, TB = LAYOUT == 3;
    constexpr int PD = NBW == 1 ? 8 : NBW == 2 ? 6 : 4;      // k chunks in flight per wavefront
    __shared__ float red[4][NBW * 4][kWave];

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const int r = lane % 16, g = lane / 16;
    const int kpart = wave % ks, rsub = wave / ks;
    const int64_t rg = blockIdx.x / p.tiles_n, cg = blockIdx.x % p.tiles_n;
    const int64_t m0 = (rg * (4 / ks) + rsub) * 16;
    const int64_t n0 = cg * (16 * NBW);
    const bool active = m0 < p.M;                              // wave-uniform

    // this wavefront's k range: whole chunks, the last part takes the ragged end
    const int64_t chunks = (p.K + 15) / 16;
    const int64_t per = (chunks + ks - 1) / ks;
    const int64_t kb = kpart * per * 16;
    const int64_t ke = (kb + per * 16 < p.K) ? kb + per * 16 : p.K;
    const int nfull = (active && ke > kb) ? (int)((ke - kb) / 16) : 0;
    const int tail = (active && ke > kb) ? (int)((ke - kb) % 16) : 0;

    // Rows and columns outside the matrix are fetched from the last valid one (in bounds; what they
    // feed is never stored).
    const int64_t mrow = (m0 + r < p.M) ? m0 + r : p.M - 1;
    int64_t ncol[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int64_t n = n0 + 16 * nb + r;
        ncol[nb] = n < p.N ? n : p.N - 1;
    }
    int64_t a_row = 0;                                         // element offset of the row's k = 0
    if constexpr (CONV) {
        const uint32_t mu = (uint32_t)mrow, OWu = (uint32_t)p.g.OW, OHu = (uint32_t)p.g.OH;
        const uint32_t q = mu / OWu;
        const int64_t ow = mu - q * OWu, n = q / OHu, oh = q - (uint32_t)n * OHu;
        a_row = ((n * p.g.H + oh * p.g.SH) * p.g.W + ow * p.g.SW) * p.g.C;
    } else if constexpr (!TA) {
        a_row = mrow * p.lda;
    }

    // Convolution: k -> filter tap (kh, kw) and channel c.  A lane walks its k positions chunk by
    // chunk (one position when it fetches 16 bytes, which never straddle a tap as C % 4 == 0 then;
    // four otherwise).  Chunks are loaded in ascending order, so the walk only moves forward.
    int wc[4] = {0, 0, 0, 0}, wkw[4] = {0, 0, 0, 0}, wkh[4] = {0, 0, 0, 0};
    const int cvC = (int)p.g.C, cvKW = (int)p.g.KW;
    if constexpr (CONV) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t k = (uint32_t)(kb + 4 * g + j);
            const uint32_t tap = k / (uint32_t)cvC;
            wc[j] = (int)(k - tap * (uint32_t)cvC);
            wkh[j] = (int)(tap / (uint32_t)cvKW);
            wkw[j] = (int)(tap - (uint32_t)wkh[j] * (uint32_t)cvKW);
        }
    }
    auto tap_offset = [&](int j) -> int64_t {
        return ((int64_t)wkh[j] * p.g.DH * p.g.W + (int64_t)wkw[j] * p.g.DW) * p.g.C + wc[j];
    };
    auto walk_on = [&](int j) {
        wc[j] += 16;
        while (wc[j] >= cvC) {
            wc[j] -= cvC;
            if (++wkw[j] == cvKW) { wkw[j] = 0; ++wkh[j]; }
        }
    };

    // Fetch the chunk at kc.  FULL: all 16 k lie inside the range; otherwise every element is
    // predicated on k < ke and reads as zero beyond (both operands, so that no NaN of an operand
    // leaks through a zero of the other).
    auto load = [&](DirectFrag<NBW>& f, int64_t kc, auto full_c) {
        constexpr bool FULL = decltype(full_c)::value;
        const int64_t k0 = kc + 4 * g;
        if constexpr (TA) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                f.a[j] = (FULL || k0 + j < ke) ? p.A[(k0 + j) * p.lda + mrow] : 0.f;
        } else if constexpr (CONV) {
            if (FULL && a_vec) {
                const float4 v = *reinterpret_cast<const float4*>(p.A + a_row + tap_offset(0));
                f.a[0] = v.x; f.a[1] = v.y; f.a[2] = v.z; f.a[3] = v.w;
                walk_on(0);
            } else {
                if (a_vec) {                                   // the ragged chunk of a 16-byte walker
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        f.a[j] = (k0 + j < ke) ? p.A[a_row + tap_offset(0) + j] : 0.f;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        f.a[j] = (FULL || k0 + j < ke) ? p.A[a_row + tap_offset(j)] : 0.f;
                        walk_on(j);
                    }
                }
            }
        } else {
            const float* ap = p.A + a_row + k0;
            if (FULL && a_vec) {
                const float4 v = *reinterpret_cast<const float4*>(ap);
                f.a[0] = v.x; f.a[1] = v.y; f.a[2] = v.z; f.a[3] = v.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) f.a[j] = (FULL || k0 + j < ke) ? ap[j] : 0.f;
            }
        }
        if constexpr (TB) {
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) {
                const float* bp = p.B + ncol[nb] * p.ldb + k0;
                if (FULL && b_vec) {
                    const float4 v = *reinterpret_cast<const float4*>(bp);
                    f.b[nb][0] = v.x; f.b[nb][1] = v.y; f.b[nb][2] = v.z; f.b[nb][3] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) f.b[nb][j] = (FULL || k0 + j < ke) ? bp[j] : 0.f;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool ok = FULL || k0 + j < ke;
                const float* bp = p.B + (k0 + j) * p.ldb;
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) f.b[nb][j] = ok ? bp[ncol[nb]] : 0.f;
            }
        }
    };

    floatx4 acc[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) acc[nb] = floatx4{0.f, 0.f, 0.f, 0.f};
    auto mma = [&](const DirectFrag<NBW>& f) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb)
                acc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(f.a[j], f.b[nb][j], acc[nb], 0, 0, 0);
    };

    if (nfull > 0 || tail > 0) {
        constexpr std::true_type whole{};
        constexpr std::false_type ragged{};
        DirectFrag<NBW> f[PD], ft;
#pragma unroll
        for (int s = 0; s < PD; ++s)
            if (s < nfull) load(f[s], kb + 16 * s, whole);
        // a short range has all its whole chunks in flight now: send the ragged one after them
        const bool tail_early = tail > 0 && nfull <= PD;
        if (tail_early) load(ft, kb + 16 * (int64_t)nfull, ragged);
        int c0 = 0;
        for (; c0 + 2 * PD <= nfull; c0 += PD) {
#pragma unroll
            for (int s = 0; s < PD; ++s) {
                mma(f[s]);
                load(f[s], kb + 16 * (int64_t)(c0 + s + PD), whole);
            }
        }
        const int rem = nfull - c0;                            // < 2 * PD chunks left, min(rem, PD) in flight
#pragma unroll
        for (int s = 0; s < PD; ++s) {
            if (s < rem) {
                mma(f[s]);
                if (s + PD < rem) load(f[s], kb + 16 * (int64_t)(c0 + s + PD), whole);
            }
        }
#pragma unroll
        for (int s = 0; s < PD; ++s)
            if (s + PD < rem) mma(f[s]);
        if (tail > 0) {
            if (!tail_early) load(ft, kb + 16 * (int64_t)nfull, ragged);
            mma(ft);
        }
    }

    // partial sums of the k parts: part 0 adds parts 1 .. ks-1 in that order
    if (ks > 1) {
        if (kpart > 0) {
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
                for (int i = 0; i < 4; ++i) red[wave][nb * 4 + i][lane] = acc[nb][i];
        }
        __syncthreads();
        if (kpart == 0) {
            for (int q = 1; q < ks; ++q)
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[nb][i] += red[wave + q][nb * 4 + i][lane];
        }
    }
    if (!active || kpart != 0) return;
    // accumulator register i of a lane is C[m0 + 4g + i][n0 + 16 nb + lane % 16]
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + 4 * g + i;
        if (m >= p.M) continue;
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            const int64_t n = n0 + 16 * nb + r;
            if (n >= p.N) continue;
            float* cp = p.C + m * p.ldc + n;
            *cp = p.accumulate ? *cp + acc[nb][i] : acc[nb][i];
        }
    }
}

template <int LAYOUT>
static int launch_direct_layout(GemmArgs a, int nbw, int ks, bool a_vec, bool b_vec, hipStream_t s) {
    const int64_t row_groups = cdiv(cdiv(a.M, 16), 4 / ks);
    const int64_t col_groups = cdiv(a.N, 16 * nbw);
    if (row_groups * col_groups > kMaxGrid) return LG_ERR_UNSUPPORTED;
    a.tiles_m = (unsigned)row_groups;
    a.tiles_n = (unsigned)col_groups;
    const dim3 grid((unsigned)(row_groups * col_groups)), block(256);
    switch (nbw) {
        case 1: hipLaunchKernelGGL((gemm_direct_kernel<LAYOUT, 1>), grid, block, 0, s, a, ks, (int)a_vec, (int)b_vec); break;
        case 2: hipLaunchKernelGGL((gemm_direct_kernel<LAYOUT, 2>), grid, block, 0, s, a, ks, (int)a_vec, (int)b_vec); break;
        default: hipLaunchKernelGGL((gemm_direct_kernel<LAYOUT, 4>), grid, block, 0, s, a, ks, (int)a_vec, (int)b_vec); break;
    }
    return launch_status();
}

int launch_direct(const GemmArgs& a, Layout layout, int nbw, int ks, hipStream_t s) {
    if ((nbw != 1 && nbw != 2 && nbw != 4) || (ks != 1 && ks != 2 && ks != 4)) return LG_ERR_INVALID_ARG;
    switch (layout) {
        case Layout::NN:
            return launch_direct_layout<0>(a, nbw, ks, a.lda % 4 == 0 && aligned16(a.A), false, s);
        case Layout::CONV:
            return launch_direct_layout<1>(a, nbw, ks, a.g.C % 4 == 0 && aligned16(a.A), false, s);
        case Layout::TN:
            return launch_direct_layout<2>(a, nbw, ks, false, false, s);
        default:
            return launch_direct_layout<3>(a, nbw, ks, a.lda % 4 == 0 && aligned16(a.A),
                                           a.ldb % 4 == 0 && aligned16(a.B), s);
    }
}

}  // namespace lg
