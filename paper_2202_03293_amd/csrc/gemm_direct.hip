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

// LAYOUT: 0 = AB, 1 = convolution, 2 = A^T B, 3 = A B^T.  AVEC: A may be fetched 16 bytes at a time
// along k (base and row pitch 16-byte aligned; convolution: C a multiple of 4); BCVEC: the same for
// B and C along their contiguous axis (N a multiple of 4 as well); otherwise every access to that
// operand is one float.  Compile-time switches on purpose: a run-time test inside the fetch splits
// it into basic blocks, and the compiler then waits for all loads in flight at every join.  A
// convolution over three channels into a multiple of four filters is the (false, true) case.
// Convolutions with K = KH*KW*C up to kTapTable get the byte offset of every k from the row's tap
// (0, 0), channel 0 as a table from the host (through the kernel arguments into LDS) instead of
// walking (kh, kw, c) per lane: the walk starts with integer divisions, which at three channels
// cost more instructions than the loads and multiplies of the whole block.
// Division of a row index (< 2^31) by an extent known on the host: q = (m * magic) >> shift, exact
// for shift = 31 + ceil(log2 d), magic = floor(2^shift / d) + 1 (the error term m / 2^shift stays
// below 1/d).  Two multiplies instead of the ~40 instructions of a 32-bit integer division.
struct FastDiv { uint32_t magic, shift; };
struct ConvDiv { FastDiv ow, oh; };                            // row m -> (n, oh, ow)
inline FastDiv make_fastdiv(int64_t d) {
    uint32_t L = 0;
    while (((int64_t)1 << L) < d) ++L;
    const uint32_t shift = 31 + L;
    const uint64_t magic = (uint64_t)(((__uint128_t)1 << shift) / (uint64_t)d) + 1;
    return FastDiv{(uint32_t)magic, magic <= 0xFFFFFFFFull ? shift : 0u};   // shift 0: no magic fits, divide
}
__device__ __forceinline__ uint32_t fastdiv(uint32_t m, const FastDiv& f, uint32_t d) {
    return f.shift ? (uint32_t)(((uint64_t)m * f.magic) >> f.shift) : m / d;
}

constexpr int kTapTable = 512;
struct DirectTaps { uint32_t off[kTapTable + 16]; };          // + one chunk of zeros for lanes past K

template <int LAYOUT, int NBW, bool AVEC, bool BCVEC, bool TABLE>
__device__ __forceinline__ void gemm_direct_body(const GemmArgs& p, int ks, const uint32_t* taps, const ConvDiv& dv,
                                                 unsigned bid) {
    constexpr bool CONV = LAYOUT == 1, TA = LAYOUT == 2, TB = LAYOUT == 3;
    static_assert(!TABLE || CONV, "the tap table belongs to the convolution");
    constexpr int PD = (BCVEC || NBW == 1) ? 4 : 2;             // k chunks per register set (one-float loads take an offset register each)
    __shared__ float red[4][NBW * 4][kWave];

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const int r = lane % 16, g = lane / 16;
    const int kpart = wave % ks, rsub = wave / ks;
    const int64_t rg = bid / p.tiles_n, cg = bid % p.tiles_n;
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
    // feed is never stored).  Block nb of a lane owns column n0 + NBW*c + nb (c = lane % 16): the
    // NBW columns of a lane are neighbours in memory, one vector load or store wide.
    const int64_t mrow = (m0 + r < p.M) ? m0 + r : p.M - 1;
    int64_t ncol[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int64_t n = n0 + NBW * r + nb;
        ncol[nb] = n < p.N ? n : p.N - 1;
    }
    // whole groups of NBW columns lie inside or outside the matrix when N % NBW == 0
    constexpr bool row_vec = NBW > 1 && BCVEC;
    const int64_t ngroup = (n0 + NBW * r < p.N) ? n0 + NBW * r : p.N - NBW;   // used when row_vec

    // Addresses are a wave-uniform base that advances by one chunk (16 k) per fetch -- chunks are
    // fetched in ascending order -- plus a per-lane 32-bit byte offset that never changes: scalar
    // adds per chunk, no vector ALU work and one register per distinct offset.  (The host sends
    // operands of 4 GiB or more to the tiled kernel.)
    const char* a_s = reinterpret_cast<const char*>(p.A);
    const char* b_s = reinterpret_cast<const char*>(p.B);
    int64_t a_step, b_step;
    uint32_t a_voff[TA ? 4 : 1];
    uint32_t b_voff[TB ? NBW : 4];
    if constexpr (CONV) {
        const uint32_t mu = (uint32_t)mrow, OWu = (uint32_t)p.g.OW, OHu = (uint32_t)p.g.OH;
        const uint32_t q = fastdiv(mu, dv.ow, OWu);
        const int64_t ow = mu - q * OWu, n = fastdiv(q, dv.oh, OHu), oh = q - (uint32_t)n * OHu;
        a_voff[0] = (uint32_t)((((n * p.g.H + oh * p.g.SH) * p.g.W + ow * p.g.SW) * p.g.C) * 4);   // tap (0, 0), channel 0
        a_step = 0;
    } else if constexpr (TA) {
        a_s += kb * p.lda * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) a_voff[j] = (uint32_t)(((4 * g + j) * p.lda + mrow) * 4);
        a_step = 64 * p.lda;
    } else {
        a_s += kb * 4;
        a_voff[0] = (uint32_t)((mrow * p.lda + 4 * g) * 4);
        a_step = 64;
    }
    if constexpr (TB) {
        b_s += kb * 4;
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) b_voff[nb] = (uint32_t)((ncol[nb] * p.ldb + 4 * g) * 4);
        b_step = 64;
    } else {
        b_s += kb * p.ldb * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) b_voff[j] = (uint32_t)(((4 * g + j) * p.ldb + (row_vec ? ngroup : 0)) * 4);
        b_step = 64 * p.ldb;
    }
    uint32_t ncol4[NBW];                                       // column byte offsets for the one-float path
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) ncol4[nb] = (uint32_t)(ncol[nb] * 4);
    int64_t kcur = kb + 4 * g;                                 // the lane's first k of the next chunk
    auto ldf = [](const char* base, uint32_t off) { return *reinterpret_cast<const float*>(base + off); };
    auto ldf4 = [](const char* base, uint32_t off) { return *reinterpret_cast<const float4*>(base + off); };

    // Convolution: k -> filter tap (kh, kw) and channel c.  A lane walks its k positions chunk by
    // chunk (one position when it fetches 16 bytes, which never straddle a tap as C % 4 == 0 then;
    // four otherwise).
    int wc[4] = {0, 0, 0, 0}, wkw[4] = {0, 0, 0, 0}, wkh[4] = {0, 0, 0, 0};
    const int cvC = (int)p.g.C, cvKW = (int)p.g.KW;
    if constexpr (CONV && !TABLE) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t k = (uint32_t)(kb + 4 * g + j);
            const uint32_t tap = k / (uint32_t)cvC;
            wc[j] = (int)(k - tap * (uint32_t)cvC);
            wkh[j] = (int)(tap / (uint32_t)cvKW);
            wkw[j] = (int)(tap - (uint32_t)wkh[j] * (uint32_t)cvKW);
        }
    }
    const uint32_t tap_kh = (uint32_t)(p.g.DH * p.g.W * p.g.C * 4), tap_kw = (uint32_t)(p.g.DW * p.g.C * 4);
    auto tap_offset = [&](int j) -> uint32_t {                 // bytes from the row's tap (0, 0), channel 0
        if constexpr (TABLE) return taps[kcur + j];
        else return (uint32_t)wkh[j] * tap_kh + (uint32_t)wkw[j] * tap_kw + (uint32_t)wc[j] * 4u;
    };
    auto walk_on = [&](int j) {
        if constexpr (TABLE) return;
        wc[j] += 16;
        while (wc[j] >= cvC) {
            wc[j] -= cvC;
            if (++wkw[j] == cvKW) { wkw[j] = 0; ++wkh[j]; }
        }
    };

    // Fetch the next chunk.  FULL: all 16 k lie inside the range; otherwise every element is
    // predicated on k < ke and reads as zero beyond (both operands, so that no NaN of an operand
    // leaks through a zero of the other).
    auto load = [&](DirectFrag<NBW>& f, auto full_c) {
        constexpr bool FULL = decltype(full_c)::value;
        if constexpr (CONV) {
            if constexpr (AVEC) {
                const uint32_t off = a_voff[0] + tap_offset(0);
                if constexpr (FULL) {
                    const float4 v = ldf4(a_s, off);
                    f.a[0] = v.x; f.a[1] = v.y; f.a[2] = v.z; f.a[3] = v.w;
                    walk_on(0);
                } else {                                       // the ragged chunk of a 16-byte walker
#pragma unroll
                    for (int j = 0; j < 4; ++j) f.a[j] = (kcur + j < ke) ? ldf(a_s, off + 4 * j) : 0.f;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f.a[j] = (FULL || kcur + j < ke) ? ldf(a_s, a_voff[0] + tap_offset(j)) : 0.f;
                    walk_on(j);
                }
            }
        } else if constexpr (TA) {
#pragma unroll
            for (int j = 0; j < 4; ++j) f.a[j] = (FULL || kcur + j < ke) ? ldf(a_s, a_voff[j]) : 0.f;
        } else {
            if constexpr (FULL && AVEC) {
                const float4 v = ldf4(a_s, a_voff[0]);
                f.a[0] = v.x; f.a[1] = v.y; f.a[2] = v.z; f.a[3] = v.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) f.a[j] = (FULL || kcur + j < ke) ? ldf(a_s, a_voff[0] + 4 * j) : 0.f;
            }
        }
        a_s += a_step;
        if constexpr (TB) {
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) {
                if constexpr (FULL && BCVEC) {
                    const float4 v = ldf4(b_s, b_voff[nb]);
                    f.b[nb][0] = v.x; f.b[nb][1] = v.y; f.b[nb][2] = v.z; f.b[nb][3] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) f.b[nb][j] = (FULL || kcur + j < ke) ? ldf(b_s, b_voff[nb] + 4 * j) : 0.f;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool ok = FULL || kcur + j < ke;
                if constexpr (row_vec && NBW == 4) {
                    const float4 v = ok ? ldf4(b_s, b_voff[j]) : make_float4(0.f, 0.f, 0.f, 0.f);
                    f.b[0][j] = v.x; f.b[1][j] = v.y; f.b[2][j] = v.z; f.b[3][j] = v.w;
                } else if constexpr (row_vec && NBW == 2) {
                    const float2 v = ok ? *reinterpret_cast<const float2*>(b_s + b_voff[j]) : make_float2(0.f, 0.f);
                    f.b[0][j] = v.x; f.b[1][j] = v.y;
                } else {
#pragma unroll
                    for (int nb = 0; nb < NBW; ++nb) f.b[nb][j] = ok ? ldf(b_s, b_voff[j] + ncol4[nb]) : 0.f;
                }
            }
        }
        b_s += b_step;
        kcur += 16;
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

    {
        constexpr std::true_type whole{};
        constexpr std::false_type ragged{};
        // Two register sets of PD chunks each.  While one set is multiplied the other is in flight, so
        // every wait is for loads issued a whole set of multiplies earlier.  (Refilling chunk by
        // chunk would keep more loads in flight, but the compiler's wait insertion then drains
        // everything at the head of the loop; with whole sets the drain it inserts there is the
        // wait that is needed anyway.)
        DirectFrag<NBW> f0[PD], f1[PD], ft;
        auto load_set = [&](DirectFrag<NBW>* f) {
#pragma unroll
            for (int s = 0; s < PD; ++s) load(f[s], whole);
            __builtin_amdgcn_sched_barrier(0);
        };
        auto mma_set = [&](const DirectFrag<NBW>* f) {
#pragma unroll
            for (int s = 0; s < PD; ++s) mma(f[s]);
            __builtin_amdgcn_sched_barrier(0);
        };
        const int sets = nfull / PD;
        int left = nfull;                                      // whole chunks not yet loaded
        if (sets >= 2) {
            load_set(f0);
            int done = 0;                                      // sets multiplied; set `done` is in flight in f0
            while (done + 2 < sets) {
                load_set(f1);
                mma_set(f0);
                load_set(f0);
                mma_set(f1);
                done += 2;
            }
            if (done + 1 < sets) {
                load_set(f1);
                mma_set(f0);
                mma_set(f1);
            } else {
                mma_set(f0);
            }
            left = nfull - sets * PD;                          // < PD
        }
        // What is left (fewer than 2*PD whole chunks, then the ragged one): all in flight at once,
        // then multiplied.
#pragma unroll
        for (int s = 0; s < PD; ++s)
            if (s < left) load(f0[s], whole);
#pragma unroll
        for (int s = 0; s < PD; ++s)
            if (s + PD < left) load(f1[s], whole);
        if (tail > 0) load(ft, ragged);
#pragma unroll
        for (int s = 0; s < PD; ++s)
            if (s < left) mma(f0[s]);
#pragma unroll
        for (int s = 0; s < PD; ++s)
            if (s + PD < left) mma(f1[s]);
        if (tail > 0) mma(ft);
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
    // accumulator register i of block nb is C[m0 + 4g + i][n0 + NBW*(lane % 16) + nb]
    constexpr bool out_vec = NBW > 1 && BCVEC;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + 4 * g + i;
        if (m >= p.M) continue;
        float* cp = p.C + m * p.ldc + n0 + NBW * r;
        if (out_vec) {
            if (n0 + NBW * r >= p.N) continue;
            if constexpr (NBW == 4) {
                float4 v = make_float4(acc[0][i], acc[1][i], acc[2][i], acc[3][i]);
                if (p.accumulate) {
                    const float4 o = *reinterpret_cast<const float4*>(cp);
                    v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                }
                *reinterpret_cast<float4*>(cp) = v;
            } else if constexpr (NBW == 2) {
                float2 v = make_float2(acc[0][i], acc[1][i]);
                if (p.accumulate) {
                    const float2 o = *reinterpret_cast<const float2*>(cp);
                    v.x += o.x; v.y += o.y;
                }
                *reinterpret_cast<float2*>(cp) = v;
            }
        } else {
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) {
                if (n0 + NBW * r + nb >= p.N) continue;
                cp[nb] = p.accumulate ? cp[nb] + acc[nb][i] : acc[nb][i];
            }
        }
    }
}

// LOOP: the grid is a fixed number of workgroups that stride over the blocks (many rounds of
// blocks: the start-up -- and the convolution's table -- are paid once per workgroup instead of
// once per block); otherwise one workgroup per group of blocks.
template <int LAYOUT, int NBW, bool AVEC, bool BCVEC, bool LOOP = false>
__global__ __launch_bounds__(256, NBW == 1 ? 4 : NBW == 2 ? 3 : 2) void gemm_direct_kernel(GemmArgs p, int ks, ConvDiv dv) {
    if constexpr (LOOP) {
        const unsigned nblocks = p.tiles_m * p.tiles_n;
        for (unsigned bid = blockIdx.x; bid < nblocks; bid += gridDim.x) {
            gemm_direct_body<LAYOUT, NBW, AVEC, BCVEC, false>(p, ks, nullptr, dv, bid);
            if (ks > 1) __syncthreads();           // the next block reuses the LDS of the k-part sums
        }
    } else {
        gemm_direct_body<LAYOUT, NBW, AVEC, BCVEC, false>(p, ks, nullptr, dv, blockIdx.x);
    }
}

template <int NBW, bool AVEC, bool BCVEC, bool LOOP>
__global__ __launch_bounds__(256, NBW == 1 ? 4 : NBW == 2 ? 3 : 2) void gemm_direct_conv_table_kernel(
    GemmArgs p, int ks, ConvDiv dv, DirectTaps host_taps) {
    __shared__ uint32_t taps[kTapTable + 16];
    for (int i = threadIdx.x; i < kTapTable + 16; i += 256) taps[i] = host_taps.off[i];
    __syncthreads();
    if constexpr (LOOP) {
        const unsigned nblocks = p.tiles_m * p.tiles_n;
        for (unsigned bid = blockIdx.x; bid < nblocks; bid += gridDim.x) {
            gemm_direct_body<1, NBW, AVEC, BCVEC, true>(p, ks, taps, dv, bid);
            if (ks > 1) __syncthreads();           // the next block reuses the LDS of the k-part sums
        }
    } else {
        gemm_direct_body<1, NBW, AVEC, BCVEC, true>(p, ks, taps, dv, blockIdx.x);
    }
}

// a_vec / bc_vec: see the kernel.  The mixed case exists for the convolution only (three input
// channels, aligned filter and output); elsewhere an unaligned A sends everything down the
// one-float path.
template <int LAYOUT>
static int launch_direct_layout(GemmArgs a, int nbw, int ks, bool a_vec, bool bc_vec, hipStream_t s) {
    const int64_t row_groups = cdiv(cdiv(a.M, 16), 4 / ks);
    const int64_t col_groups = cdiv(a.N, 16 * nbw);
    if (row_groups * col_groups > kMaxGrid) return LG_ERR_UNSUPPORTED;
    a.tiles_m = (unsigned)row_groups;
    a.tiles_n = (unsigned)col_groups;
    const int64_t nblocks = row_groups * col_groups;
    const dim3 grid((unsigned)nblocks), block(256);
    ConvDiv dv{};
    if constexpr (LAYOUT == 1) dv = ConvDiv{make_fastdiv(a.g.OW), make_fastdiv(a.g.OH)};
    if constexpr (LAYOUT == 1) {
        if (a.K <= kTapTable) {
            DirectTaps taps{};
            for (int64_t k = 0; k < a.K; ++k) {
                const int64_t c = k % a.g.C, tap = k / a.g.C, kw = tap % a.g.KW, kh = tap / a.g.KW;
                taps.off[k] = (uint32_t)(((kh * a.g.DH * a.g.W + kw * a.g.DW) * a.g.C + c) * 4);
            }
            // many rounds of blocks (and aligned filter/output, the case this is for): as many
            // workgroups as the chip holds at once -- 4 / 3 / 2 per SIMD by the register budget --
            // each striding over the blocks
            const int64_t resident = (int64_t)kCUs * (nbw == 1 ? 4 : nbw == 2 ? 3 : 2);
            const bool loop = bc_vec && nblocks > 4 * resident;
            const dim3 lgrid((unsigned)resident);
#define LG_DIRECT_TABLE(NBW)                                                                                                 \
    do {                                                                                                                     \
        if (loop && a_vec)   hipLaunchKernelGGL((gemm_direct_conv_table_kernel<NBW, true, true, true>), lgrid, block, 0, s, a, ks, dv, taps);   \
        else if (loop)       hipLaunchKernelGGL((gemm_direct_conv_table_kernel<NBW, false, true, true>), lgrid, block, 0, s, a, ks, dv, taps);  \
        else if (a_vec && bc_vec) hipLaunchKernelGGL((gemm_direct_conv_table_kernel<NBW, true, true, false>), grid, block, 0, s, a, ks, dv, taps);   \
        else if (bc_vec)     hipLaunchKernelGGL((gemm_direct_conv_table_kernel<NBW, false, true, false>), grid, block, 0, s, a, ks, dv, taps);  \
        else                 hipLaunchKernelGGL((gemm_direct_conv_table_kernel<NBW, false, false, false>), grid, block, 0, s, a, ks, dv, taps); \
    } while (0)
            switch (nbw) {
                case 1: LG_DIRECT_TABLE(1); break;
                case 2: LG_DIRECT_TABLE(2); break;
                default: LG_DIRECT_TABLE(4); break;
            }
#undef LG_DIRECT_TABLE
            return launch_status();
        }
    }
    const bool all_vec = a_vec && bc_vec;
    if constexpr (LAYOUT == 0) {
        // AB with aligned B and C over many rounds of blocks (a tall matrix times a small one): the
        // striding grid, and the mixed case of an A whose rows are not 16-byte aligned
        const int64_t resident = (int64_t)kCUs * (nbw == 1 ? 4 : nbw == 2 ? 3 : 2);
        if (bc_vec && nblocks > 4 * resident) {
            const dim3 lgrid((unsigned)resident);
#define LG_DIRECT_LOOP(NBW)                                                                                                  \
    do {                                                                                                                     \
        if (a_vec) hipLaunchKernelGGL((gemm_direct_kernel<0, NBW, true, true, true>), lgrid, block, 0, s, a, ks, dv);        \
        else       hipLaunchKernelGGL((gemm_direct_kernel<0, NBW, false, true, true>), lgrid, block, 0, s, a, ks, dv);       \
    } while (0)
            switch (nbw) {
                case 1: LG_DIRECT_LOOP(1); break;
                case 2: LG_DIRECT_LOOP(2); break;
                default: LG_DIRECT_LOOP(4); break;
            }
#undef LG_DIRECT_LOOP
            return launch_status();
        }
    }
#define LG_DIRECT(NBW)                                                                                              \
    do {                                                                                                            \
        if (all_vec) hipLaunchKernelGGL((gemm_direct_kernel<LAYOUT, NBW, true, true>), grid, block, 0, s, a, ks, dv);   \
        else         hipLaunchKernelGGL((gemm_direct_kernel<LAYOUT, NBW, false, false>), grid, block, 0, s, a, ks, dv); \
    } while (0)
    switch (nbw) {
        case 1: LG_DIRECT(1); break;
        case 2: LG_DIRECT(2); break;
        default: LG_DIRECT(4); break;
    }
#undef LG_DIRECT
    return launch_status();
}

// The kernel addresses its operands with 32-bit byte offsets.
bool direct_can_run(const GemmArgs& a, Layout layout) {
    const int64_t lim = (int64_t)1 << 32, ld_lim = (int64_t)1 << 26;
    int64_t a_bytes, b_bytes;
    switch (layout) {
        case Layout::CONV: a_bytes = a.M / (a.g.OH * a.g.OW) * a.g.H * a.g.W * a.g.C * 4; break;
        case Layout::TN: a_bytes = ((a.K - 1) * a.lda + a.M) * 4; break;
        default: a_bytes = ((a.M - 1) * a.lda + a.K) * 4; break;
    }
    b_bytes = layout == Layout::NT ? ((a.N - 1) * a.ldb + a.K) * 4 : ((a.K - 1) * a.ldb + a.N) * 4;
    return a_bytes < lim && b_bytes < lim && a.lda < ld_lim && a.ldb < ld_lim;
}

// Alignment verdicts, per operand (the tiled kernel's single verdict also wants K a multiple of 4,
// which whole 16-deep chunks do not need).
int launch_direct(const GemmArgs& a, Layout layout, int nbw, int ks, hipStream_t s) {
    if ((nbw != 1 && nbw != 2 && nbw != 4) || (ks != 1 && ks != 2 && ks != 4)) return LG_ERR_INVALID_ARG;
    if (!direct_can_run(a, layout)) return LG_ERR_UNSUPPORTED;
    const bool c_ok = a.ldc % 4 == 0 && a.N % 4 == 0 && aligned16(a.C);
    const bool a_row_ok = a.lda % 4 == 0 && aligned16(a.A);
    const bool b_row_ok = a.ldb % 4 == 0 && aligned16(a.B);
    switch (layout) {
        case Layout::NN: return launch_direct_layout<0>(a, nbw, ks, a_row_ok, b_row_ok && c_ok, s);
        case Layout::CONV: return launch_direct_layout<1>(a, nbw, ks, a.g.C % 4 == 0 && aligned16(a.A), b_row_ok && c_ok, s);
        case Layout::TN: return launch_direct_layout<2>(a, nbw, ks, b_row_ok && c_ok, b_row_ok && c_ok, s);   // A is never fetched along k
        default: return launch_direct_layout<3>(a, nbw, ks, a_row_ok, b_row_ok && c_ok, s);
    }
}

}  // namespace lg
