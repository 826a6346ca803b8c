// Matmul (Section 4.6.1, equation AB) and conv_2d_nhwc_hwcf (Section 4.6.2) on the fp32 matrix
// cores of gfx950.  One kernel template serves both: the convolution is the same contraction with
// M = N*OH*OW, N = F, K = KH*KW*C, whose A operand is gathered from the NHWC input on the fly
// (implicit GEMM; the HWCF filter already is a row-major [K, F] matrix).
//
// Decomposition (the hardware counterpart of the paper's tile / pack / vectorise / contract steps):
//   grid      -> BM x BN output tiles, dealt so that each XCD's L2 sees a compact block of tiles
//   workgroup -> stages A[BM x BK] and B[BK x BN] k-slices global -> LDS directly (no registers), a ring
//                of three LDS stages with the transfers running two slices ahead of the multiply
//   wavefront -> WM x WN register tile of 32x32 fp32 accumulators, v_mfma_f32_32x32x2_f32
//   epilogue  -> accumulators (+ C) straight to global memory with 128-bit stores
//
// Operand placement tricks that rely only on the sum over k and the set of columns being
// order-free:
//   * k-permutation: the two half-waves of an MFMA hold k and k' of a pair; a lane reads FOUR
//     consecutive k of its A row with one ds_read_b128 and feeds them to four MFMAs, while the B
//     rows are picked to match (half h of step 4j+i uses k = 8j + 4h + i).
//   * n-interleave: column block nb of a wave tile holds columns NB*c + nb (c = lane % 32), so one
//     ds_read_b{32*NB} fetches the B values of all NB blocks and the epilogue finds NB adjacent
//     columns of one row in one lane -> 128-bit stores when NB = 4.
#include "lg_common.hpp"
#include <type_traits>

namespace lg {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void;

// LDS byte address of a pointer into __shared__ memory.
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(lds_void*)p;
}

// One global -> LDS transfer of 16 bytes per lane: lane l's data lands at LDS address lds + 16*l.
// `base` and `lds` must be wave-uniform; `voff` is the lane's byte offset from base.  Written as
// inline assembly on purpose: the compiler then neither knows that LDS is being written
// asynchronously (it would otherwise make every later ds_read wait for ALL transfers in flight,
// defeating the prefetch) nor orders anything around it, so the caller owns the synchronisation:
// dma_wait<N>() followed by a workgroup barrier before the data is read.
__device__ __forceinline__ void dma16(const void* base, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds), "v"(voff), "s"(base) : "memory");
}

// Wait until at most N of this wave's global->LDS transfers are still in flight.
template <int N>
__device__ __forceinline__ void dma_wait() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

struct ConvGeom {        // implicit-GEMM A operand: row m -> (n, oh, ow), column k -> (kh, kw, c)
    int64_t H, W, C, KW, SH, SW, DH, DW, OH, OW;
};

struct GemmArgs {
    const float* A;      // matmul: M x K, row stride lda.  conv: NHWC input
    const float* B;      // K x N, row stride ldb
    float* C;            // M x N, row stride ldc (or split-k partials: slab z at C + z*M*ldc)
    int64_t M, N, K;
    int64_t lda, ldb, ldc;
    int64_t k_per_split; // multiple of the tile's BK; slab z covers k in [z*k_per_split, min(K, (z+1)*k_per_split))
    int accumulate;      // only honoured when the grid has one k-slab
    unsigned tiles_m, tiles_n;
    ConvGeom g;
};

// BM x BN output tile per workgroup, BK-deep k-slices, WM x WN register tile per wavefront.
// MINW = wavefronts per SIMD the register allocation must leave room for.
template <int BM_, int BN_, int BK_, int WM_, int WN_, int MINW_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MINW = MINW_;
    static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
    static constexpr int WAVES = WAVES_M * WAVES_N;
    static constexpr int THREADS = WAVES * kWave;
    static constexpr int MB = WM / 32;              // accumulator blocks along m per wave
    static constexpr int NB = WN / 32;              // along n (1, 2 or 4: lanes hold NB adjacent columns)
    static constexpr int QPR = BK / 4;              // float4s per A row of a slice
    static constexpr int A_QUADS = BM * BK / 4;     // float4s in an A slice
    static constexpr int B_QUADS = BK * BN / 4;
    static constexpr int A_PER_T = A_QUADS / THREADS;
    static constexpr int B_PER_T = B_QUADS / THREADS;
    static constexpr int A_ROW_STEP = THREADS / QPR;
    static constexpr int STAGES = 3;                // LDS ring: one slice being multiplied, two in flight
    static constexpr int LDS_FLOATS = STAGES * (BM * BK + BK * BN);
    static_assert(BK == 16 || BK == 32 || BK == 64, "k-slice depth");
    static_assert(NB == 1 || NB == 2 || NB == 4, "wave tile width must be 32, 64 or 128");
    static_assert(A_QUADS % THREADS == 0 && B_QUADS % THREADS == 0, "slice must divide over the workgroup");
    static_assert(THREADS % QPR == 0, "A staging layout");
    static_assert(A_PER_T == 1 || A_ROW_STEP % 8 == 0, "a lane's A rows must share one swizzle");

    // LDS position (in floats) of the float4 holding A[m][4q .. 4q+3] of a slice.  Rows are BK floats;
    // the quad index is XOR-swizzled with bits of m so that 8 consecutive rows reading the same
    // logical quad touch 8 distinct 4-bank groups (and so do the 8 lanes that write a row pair / row).
    // swizzle(m): 3 (or 2) row bits XOR-ed into the quad index.  A row is BK floats = BK/32 times all
    // banks (BK = 16: two rows span the banks, so the row bits used start at bit 1).
    static constexpr int SWZ_SH = (QPR == 4) ? 1 : 0;
    static constexpr int SWZ_MASK = (QPR < 8) ? QPR - 1 : 7;
    __device__ static __forceinline__ int swizzle(int m) { return (m >> SWZ_SH) & SWZ_MASK; }
    __device__ static __forceinline__ int a_off(int m, int q) { return m * BK + ((q ^ swizzle(m)) << 2); }
};

template <class T, bool VEC, bool CONV>
__global__ __launch_bounds__(T::THREADS, T::MINW) void gemm_kernel(const GemmArgs p) {
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, MB = T::MB, NB = T::NB;
    extern __shared__ __align__(16) float lds[];
    float* As = lds;                               // [STAGES][BM*BK]
    float* Bs = lds + T::STAGES * BM * BK;         // [STAGES][BK*BN]

    // ---- which tile ------------------------------------------------------------------------
    const unsigned ntiles = p.tiles_m * p.tiles_n;
    const unsigned L = xcd_contiguous_id(blockIdx.x, ntiles);
    constexpr unsigned GM = 8;              // tile rows per panel: the ~64 workgroups an XCD runs at once form an 8 x 8 block of tiles
    const unsigned panel = L / (GM * p.tiles_n);
    const unsigned first_m = panel * GM;
    const unsigned gsz = (p.tiles_m - first_m < GM) ? p.tiles_m - first_m : GM;
    const unsigned in_panel = L - panel * GM * p.tiles_n;
    const int64_t m0 = (int64_t)(first_m + in_panel % gsz) * BM;
    const int64_t n0 = (int64_t)(in_panel / gsz) * BN;
    const int64_t kbeg = (int64_t)blockIdx.y * p.k_per_split;
    const int64_t kend = (kbeg + p.k_per_split < p.K) ? kbeg + p.k_per_split : p.K;
    const int nslices = (int)((kend - kbeg + BK - 1) / BK);

    const int t = threadIdx.x;
    const int lane = t % kWave, wave = t / kWave;
    const int wm0 = (wave / T::WAVES_N) * T::WM;   // wave tile origin inside the block tile
    const int wn0 = (wave % T::WAVES_N) * T::WN;
    const int c32 = lane % 32, h = lane / 32;

    // ---- global -> register staging coordinates ---------------------------------------------------
    // A slice: this lane owns the float4 (row t/QPR + i*A_ROW_STEP, quad aq); B slice: float4 number
    // t + i*THREADS of the row-major [BK][BN] slice.
    const int aq = t % T::QPR;
    const int ar0 = t / T::QPR;
    int64_t a_rowbase[T::A_PER_T];          // element offset of A[m][0]; -1 when the row is outside M
#pragma unroll
    for (int i = 0; i < T::A_PER_T; ++i) {
        const int64_t m = m0 + ar0 + i * T::A_ROW_STEP;
        if (m >= p.M) { a_rowbase[i] = -1; continue; }
        if constexpr (CONV) {
            const int64_t ow = m % p.g.OW, oh = (m / p.g.OW) % p.g.OH, n = m / (p.g.OW * p.g.OH);
            a_rowbase[i] = ((n * p.g.H + oh * p.g.SH) * p.g.W + ow * p.g.SW) * p.g.C;
        } else {
            a_rowbase[i] = m * p.lda;
        }
    }
    float4 ra[T::A_PER_T], rb[T::B_PER_T];

    auto a_koff = [&](int64_t k) -> int64_t {      // offset of column k relative to the row base
        if constexpr (CONV) {
            const int64_t c = k % p.g.C, kk = k / p.g.C;
            const int64_t kw = kk % p.g.KW, kh = kk / p.g.KW;
            return (kh * p.g.DH * p.g.W + kw * p.g.DW) * p.g.C + c;
        } else {
            return k;
        }
    };

    // General slice load: every access predicated (edge tiles, k tails, unaligned operands).
    auto load_slice_edge = [&](int64_t k0) {
        if constexpr (VEC) {
            const int64_t k = k0 + 4 * aq;
            const bool kin = k < kend;             // K % 4 == 0 on this path: a quad is all in or all out
            const int64_t ko = kin ? a_koff(k) : 0;
#pragma unroll
            for (int i = 0; i < T::A_PER_T; ++i) {
                ra[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (kin && a_rowbase[i] >= 0) ra[i] = *reinterpret_cast<const float4*>(p.A + a_rowbase[i] + ko);
            }
        } else {
            int64_t ko[4];
            bool kin[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t k = k0 + 4 * aq + e;
                kin[e] = k < kend;
                ko[e] = kin[e] ? a_koff(k) : 0;
            }
#pragma unroll
            for (int i = 0; i < T::A_PER_T; ++i) {
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                if (a_rowbase[i] >= 0) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (kin[e]) v[e] = p.A[a_rowbase[i] + ko[e]];
                }
                ra[i] = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
#pragma unroll
        for (int i = 0; i < T::B_PER_T; ++i) {
            const int q = t + i * T::THREADS;
            const int kr = q / (BN / 4), nq = q % (BN / 4);
            const int64_t k = k0 + kr, n = n0 + 4 * nq;
            rb[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k < kend) {
                const float* bp = p.B + k * p.ldb + n;
                if constexpr (VEC) {
                    if (n < p.N) rb[i] = *reinterpret_cast<const float4*>(bp);   // N % 4 == 0 here
                } else {
                    if (n + 0 < p.N) rb[i].x = bp[0];
                    if (n + 1 < p.N) rb[i].y = bp[1];
                    if (n + 2 < p.N) rb[i].z = bp[2];
                    if (n + 3 < p.N) rb[i].w = bp[3];
                }
            }
        }
    };

    // Interior slices (whole tile inside M x N, whole slices inside the k-slab, aligned operands)
    // bypass the registers: global_load_lds_dwordx4 moves 16 bytes per lane straight into LDS, the
    // 64 lanes of a wave filling 1 KiB at consecutive addresses.  A and B slices are therefore laid
    // out in LDS in lane order: float4 number q = t + i*THREADS of a slice is written by lane t's
    // i-th load.  For B (row-major [BK][BN]) that is the natural order.  For A, physical quad
    // q % QPR of row q / QPR must hold the logical quad (q % QPR) ^ swizzle(row), so the lane simply
    // FETCHES that logical quad; the XOR swizzle costs nothing.  Addresses are a wave-uniform base
    // (advanced by scalar adds) plus a per-lane 32-bit byte offset that never changes.
    const char* a_base = reinterpret_cast<const char*>(p.A);
    const char* b_base = reinterpret_cast<const char*>(p.B);
    uint32_t a_loff[T::A_PER_T], b_loff[T::B_PER_T];
    // Convolution gather: this lane's quad sits at (kh, kw, c); its byte offset from the row base,
    // cv_off, is advanced incrementally.  One k-slice moves c by BK; when c passes C the tap moves on
    // (kw, then kh), which changes the offset by constants that are the same for every lane.  For
    // C >= BK at most one wrap happens per slice and the update is branch-free.
    int cv_c = 0, cv_kw = 0, cv_kh = 0;
    uint32_t cv_off = 0;
    const int lq = aq ^ T::swizzle(ar0);          // logical quad this lane fetches
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int cvC = (int)p.g.C, cvKW = (int)p.g.KW;
    const uint32_t cv_d_kw = (uint32_t)((p.g.DW * p.g.C - p.g.C) * 4);                       // c wraps, kw + 1
    const uint32_t cv_d_kh = (uint32_t)((p.g.DH * p.g.W * p.g.C - p.g.KW * p.g.DW * p.g.C) * 4);   // kw wraps, kh + 1
    auto cv_offset = [&]() {
        return (uint32_t)((((int64_t)cv_kh * p.g.DH * p.g.W + (int64_t)cv_kw * p.g.DW) * p.g.C + cv_c) * 4);
    };
    // When C is a multiple of BK a slice never straddles a filter tap, the walk is the same for all
    // lanes and lives in scalar registers (su_*): the main loop then spends no vector ALU
    // instruction on it (vector ALU instructions are not free here: they take issue slots from the
    // matrix pipe, which small tiles feel).
    const bool conv_uniform = CONV && (cvC % BK == 0);
    int su_c = 0, su_kw = 0;
    uint32_t su_off = 0;
    auto init_full = [&]() {
        if constexpr (CONV) {
            if (conv_uniform) {
                su_c = (int)(kbeg % p.g.C);
                su_kw = (int)((kbeg / p.g.C) % p.g.KW);
                const int64_t kh = kbeg / (p.g.C * p.g.KW);
                su_off = (uint32_t)(((kh * p.g.DH * p.g.W + (int64_t)su_kw * p.g.DW) * p.g.C + su_c) * 4);
#pragma unroll
                for (int i = 0; i < T::A_PER_T; ++i) a_loff[i] = (uint32_t)(a_rowbase[i] * 4) + 16u * lq;
            } else {
                const int64_t k = kbeg + 4 * lq;
                cv_c = (int)(k % p.g.C);
                cv_kw = (int)((k / p.g.C) % p.g.KW);
                cv_kh = (int)(k / (p.g.C * p.g.KW));
                cv_off = cv_offset();
#pragma unroll
                for (int i = 0; i < T::A_PER_T; ++i) a_loff[i] = (uint32_t)(a_rowbase[i] * 4);
            }
        } else {
            a_base += (m0 * p.lda + kbeg) * 4;
#pragma unroll
            for (int i = 0; i < T::A_PER_T; ++i)
                a_loff[i] = (uint32_t)(((int64_t)(ar0 + i * T::A_ROW_STEP) * p.lda + 4 * lq) * 4);
        }
        b_base += (kbeg * p.ldb + n0) * 4;
#pragma unroll
        for (int i = 0; i < T::B_PER_T; ++i) {
            const int q = t + i * T::THREADS;
            b_loff[i] = (uint32_t)(((int64_t)(q / (BN / 4)) * p.ldb + 4 * (q % (BN / 4))) * 4);
        }
    };
    // Start the transfer of the next slice into LDS stage `buf`.
    auto issue_slice = [&](int buf) {
        float* as = As + buf * (BM * BK) + 4 * 64 * wave_u;
        float* bs = Bs + buf * (BK * BN) + 4 * 64 * wave_u;
        if (CONV && conv_uniform) {
            const char* ab = a_base + su_off;
#pragma unroll
            for (int i = 0; i < T::A_PER_T; ++i) dma16(ab, a_loff[i], lds_addr(as + 4 * i * T::THREADS));
        } else {
            const uint32_t ko = CONV ? cv_off : 0u;
#pragma unroll
            for (int i = 0; i < T::A_PER_T; ++i) dma16(a_base, a_loff[i] + ko, lds_addr(as + 4 * i * T::THREADS));
        }
#pragma unroll
        for (int i = 0; i < T::B_PER_T; ++i) dma16(b_base, b_loff[i], lds_addr(bs + 4 * i * T::THREADS));
        if (CONV && conv_uniform) {
            su_c += BK;
            const bool w1 = su_c >= cvC;
            su_c -= w1 ? cvC : 0;
            su_kw += w1 ? 1 : 0;
            const bool w2 = su_kw == cvKW;
            su_kw = w2 ? 0 : su_kw;
            su_off += BK * 4 + (w1 ? cv_d_kw : 0u) + (w2 ? cv_d_kh : 0u);
        } else if constexpr (CONV) {
            cv_c += BK;
            if (cvC >= BK) {                       // uniform test; one possible wrap, no branches below
                const bool w1 = cv_c >= cvC;
                cv_c -= w1 ? cvC : 0;
                cv_kw += w1 ? 1 : 0;
                const bool w2 = cv_kw == cvKW;
                cv_kw = w2 ? 0 : cv_kw;
                cv_off += BK * 4 + (w1 ? cv_d_kw : 0u) + (w2 ? cv_d_kh : 0u);
            } else {
                while (cv_c >= cvC) {
                    cv_c -= cvC;
                    if (++cv_kw == cvKW) { cv_kw = 0; ++cv_kh; }
                }
                cv_off = cv_offset();
            }
        } else {
            a_base += BK * 4;
        }
        b_base += (int64_t)BK * p.ldb * 4;
    };

    auto store_slice = [&](int buf) {
        float* as = As + buf * (BM * BK);
        float* bs = Bs + buf * (BK * BN);
#pragma unroll
        for (int i = 0; i < T::A_PER_T; ++i)
            *reinterpret_cast<float4*>(as + T::a_off(ar0 + i * T::A_ROW_STEP, aq)) = ra[i];
#pragma unroll
        for (int i = 0; i < T::B_PER_T; ++i)
            *reinterpret_cast<float4*>(bs + 4 * (t + i * T::THREADS)) = rb[i];      // row-major [BK][BN]
    };

    // ---- accumulators ------------------------------------------------------------------------
    floatx16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

    // One k-slice from LDS.  Half-wave h of MFMA step st = 4j + i multiplies k = 8j + 4h + i.
    // Software-pipelined: all A fragments of the slice are fetched up front, the B fragment of
    // step st+1 is fetched before the MFMAs of step st are issued, so LDS latency hides behind
    // MB*NB*64 cycles of matrix work instead of stalling the in-order wave.
    auto compute_slice = [&](int buf) {
        const float* as = As + buf * (BM * BK);
        const float* bs = Bs + buf * (BK * BN) + wn0 + NB * c32 + 4 * h * BN;
        constexpr int NJ = BK / 8, NSTEP = BK / 2;
        float4 a[NJ][MB];
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                a[j][mb] = *reinterpret_cast<const float4*>(as + T::a_off(wm0 + mb * 32 + c32, 2 * j + h));
        float b[2][NB];
        auto load_b = [&](int st, float (&dst)[NB]) {
            const float* brow = bs + (8 * (st / 4) + (st % 4)) * BN;
            if constexpr (NB == 4) {
                const float4 v = *reinterpret_cast<const float4*>(brow);
                dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
            } else if constexpr (NB == 2) {
                const float2 v = *reinterpret_cast<const float2*>(brow);
                dst[0] = v.x; dst[1] = v.y;
            } else {
                dst[0] = *brow;
            }
        };
        load_b(0, b[0]);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            if (st + 1 < NSTEP) load_b(st + 1, b[(st + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            const int j = st / 4, i = st % 4;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const float av = (i == 0) ? a[j][mb].x : (i == 1) ? a[j][mb].y : (i == 2) ? a[j][mb].z : a[j][mb].w;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b[st & 1][nb], acc[mb][nb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop --------------------------------------------------------------------------
    // The interior path addresses operands with 32-bit byte offsets from the tile origin.
    const bool small_offsets = CONV ? (p.g.H * p.g.W * p.g.C * (p.M / (p.g.OH * p.g.OW) + 1) * 4 < ((int64_t)1 << 31))
                                    : ((int64_t)BM * p.lda * 4 < ((int64_t)1 << 31));
    const bool interior = VEC && small_offsets && ((int64_t)BK * p.ldb * 4 < ((int64_t)1 << 31)) &&
                          (m0 + BM <= p.M) && (n0 + BN <= p.N) && ((kend - kbeg) % BK == 0);
    if (nslices > 0) {
        if (interior) {
            // Ring of three LDS stages, transfers two slices ahead.  Each wave waits for its own
            // transfers of the slice needed next (vmcnt counts them in order), then the barrier makes
            // everybody's visible and also guarantees nobody still reads the stage refilled next.
            constexpr int L = T::A_PER_T + T::B_PER_T;      // transfers per slice per wave
            init_full();
            issue_slice(0);
            if (nslices > 1) {
                issue_slice(1);
                dma_wait<L>();
            } else {
                dma_wait<0>();
            }
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // One trip = three slices, one per LDS stage, so that every LDS address in the loop is a
            // lane constant plus an immediate (no vector ALU work per slice).
            auto step = [&](auto stage_c, int s) {
                constexpr int stage = decltype(stage_c)::value;
                if (s + 2 < nslices) issue_slice((stage + 2) % 3);
                compute_slice(stage);
                if (s + 1 < nslices) {
                    if (s + 2 < nslices) dma_wait<L>(); else dma_wait<0>();
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
            };
            int s = 0;
            for (; s + 3 <= nslices; s += 3) {
                step(std::integral_constant<int, 0>{}, s);
                step(std::integral_constant<int, 1>{}, s + 1);
                step(std::integral_constant<int, 2>{}, s + 2);
            }
            if (s < nslices) step(std::integral_constant<int, 0>{}, s);
            if (s + 1 < nslices) step(std::integral_constant<int, 1>{}, s + 1);
        } else {
            load_slice_edge(kbeg);
            store_slice(0);
            __syncthreads();
            for (int s = 0; s < nslices; ++s) {
                const bool more = s + 1 < nslices;
                if (more) load_slice_edge(kbeg + (int64_t)(s + 1) * BK);
                compute_slice(s & 1);
                if (more) store_slice((s + 1) & 1);
                __syncthreads();
            }
        }
    }

    // ---- epilogue ------------------------------------------------------------------------------
    // accumulator register r of block (mb, nb): row = 32*mb + 8*(r/4) + 4*h + r%4, column = NB*c32 + nb
    float* Cz = p.C + (int64_t)blockIdx.y * p.M * p.ldc;
    const int64_t ncol = n0 + wn0 + NB * c32;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t m = m0 + wm0 + mb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
            if (m >= p.M) continue;
            float* cp = Cz + m * p.ldc + ncol;
            float v[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) v[nb] = acc[mb][nb][r];
            if constexpr (VEC && NB == 4) {
                if (ncol < p.N) {
                    float4 o = make_float4(v[0], v[1], v[2], v[3]);
                    if (p.accumulate) {
                        const float4 c = *reinterpret_cast<const float4*>(cp);
                        o.x += c.x; o.y += c.y; o.z += c.z; o.w += c.w;
                    }
                    *reinterpret_cast<float4*>(cp) = o;
                }
            } else if constexpr (VEC && NB == 2) {
                if (ncol < p.N) {
                    float2 o = make_float2(v[0], v[1]);
                    if (p.accumulate) {
                        const float2 c = *reinterpret_cast<const float2*>(cp);
                        o.x += c.x; o.y += c.y;
                    }
                    *reinterpret_cast<float2*>(cp) = o;
                }
            } else {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    if (ncol + nb < p.N) cp[nb] = p.accumulate ? cp[nb] + v[nb] : v[nb];
            }
        }
    }
}

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

// ---- host side ---------------------------------------------------------------------------------

// The tile menu (all: 4 wavefronts, one per SIMD).  `occ` = workgroups of that tile a CU can hold
// (LDS and registers), `mfma` = matrix-pipe clocks one k-slice costs one SIMD, `eff` = the measured
// fraction of the matrix-pipe rate the tile sustains with a full CU (4096^3, clock-normalised).
using Tile0 = Tile<128, 256, 16, 64, 128, 2>;   // waves of 64x128
using Tile1 = Tile<128, 128, 16, 32, 128, 4>;   // waves of 32x128
using Tile2 = Tile<128, 64, 16, 32, 64, 4>;     // waves of 32x64 (narrow outputs, e.g. F = 64)
using Tile3 = Tile<64, 64, 16, 32, 32, 4>;      // waves of 32x32 (small problems)
using Tile4 = Tile<64, 128, 32, 32, 64, 4>;     // waves of 32x64, deeper slices (mid-size problems)
using Tile5 = Tile<64, 64, 32, 32, 32, 4>;      // waves of 32x32, deeper slices

struct TileInfo { int bm, bn, bk, occ, mfma; double eff; };
constexpr int kNumTiles = 6;
static const TileInfo kTiles[kNumTiles] = {
    {128, 256, 16, 2, 4096, 0.935}, {128, 128, 16, 4, 2048, 0.92}, {128, 64, 16, 4, 1024, 0.90},
    {64, 64, 16, 6, 512, 0.875},    {64, 128, 32, 2, 2048, 0.89},  {64, 64, 32, 3, 1024, 0.87}};

struct Plan {
    int tile;          // index into kTiles
    int64_t tiles_m, tiles_n, splits, k_per_split;
};

constexpr int kCUs = 256;
constexpr int kKGran = 64;   // split-k slabs are multiples of this (a multiple of every tile's BK)

// Pick (tile, k-split) with a cost model fitted to measurements on this part: when c workgroups
// share a CU, one k-slice of all of them takes  c * mfma / eff + dead / c  clocks, where `dead`
// (barrier skew + LDS refill after the barrier, ~350 clocks, more for deeper slices) is only
// hidden by other workgroups.  The busiest CU decides; a launch costs ~4 us of fill and drain;
// split-k adds the partial-sum traffic and a second launch.
static Plan make_plan(int64_t M, int64_t N, int64_t K) {
    const double clk = 2.4e9;
    const int64_t kslabs = cdiv(K, kKGran);
    static const int split_menu[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32};
    Plan best{};
    double best_cost = 1e300;
    for (int ti = 0; ti < kNumTiles; ++ti) {
        const TileInfo& tl = kTiles[ti];
        const int64_t tm = cdiv(M, tl.bm), tn = cdiv(N, tl.bn);
        const double dead = 350.0 + 8.0 * (tl.bk - 16);
        for (int sp : split_menu) {
            if (sp > 1 && kslabs < 2 * sp) break;                // keep at least 128 k per slab
            const int64_t kps = cdiv(kslabs, sp) * kKGran;
            const int64_t splits = cdiv(K, kps);
            if (splits != sp && sp > 1) continue;                // same plan as a smaller menu entry
            const int64_t wgs = tm * tn * splits;
            const double nslices = (double)cdiv(kps < K ? kps : K, tl.bk);
            const int64_t per_cu = cdiv(wgs, kCUs);              // workgroups on the busiest CU
            const int64_t full = per_cu / tl.occ, rest = per_cu % tl.occ;
            double clocks = (double)full * nslices * (tl.occ * tl.mfma / tl.eff + dead / tl.occ);
            if (rest) clocks += nslices * (rest * tl.mfma / tl.eff + dead / rest);
            double cost = clocks / clk + 4e-6;
            if (splits > 1) cost += 2.0 * splits * M * N * 4.0 / 3.0e12 + 5e-6;
            if (cost < best_cost) {
                best_cost = cost;
                best.tile = ti; best.tiles_m = tm; best.tiles_n = tn; best.splits = splits; best.k_per_split = kps;
            }
        }
    }
    return best;
}

static size_t plan_workspace(const Plan& pl, int64_t M, int64_t N) {
    return pl.splits > 1 ? (size_t)(pl.splits * M * N) * sizeof(float) : 0;
}

template <class T, bool VEC, bool CONV>
static void launch_gemm(const GemmArgs& a, unsigned splits, hipStream_t s) {
    static bool configured = false;
    const size_t lds_bytes = T::LDS_FLOATS * sizeof(float);
    if (!configured) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<T, VEC, CONV>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        configured = true;
    }
    hipLaunchKernelGGL((gemm_kernel<T, VEC, CONV>), dim3(a.tiles_m * a.tiles_n, splits), dim3(T::THREADS),
                       lds_bytes, s, a);
}

template <bool CONV>
static int run_gemm(GemmArgs a, bool vec, int user_accumulate, void* workspace, size_t workspace_bytes,
                    hipStream_t s) {
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
    const unsigned z = (unsigned)pl.splits;
#define LG_LAUNCH(TILE)                                                   \
    do {                                                                  \
        if (vec) launch_gemm<TILE, true, CONV>(a, z, s);                  \
        else     launch_gemm<TILE, false, CONV>(a, z, s);                 \
    } while (0)
    switch (pl.tile) {
        case 0: LG_LAUNCH(Tile0); break;
        case 1: LG_LAUNCH(Tile1); break;
        case 2: LG_LAUNCH(Tile2); break;
        case 3: LG_LAUNCH(Tile3); break;
        case 4: LG_LAUNCH(Tile4); break;
        default: LG_LAUNCH(Tile5); break;
    }
#undef LG_LAUNCH
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
    return run_gemm<false>(a, vec, accumulate, workspace, workspace_bytes, s);
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
    GemmArgs a{};
    a.A = I; a.B = Kf; a.C = O;
    a.M = M; a.N = F; a.K = Kg;
    a.lda = 0; a.ldb = F; a.ldc = F;
    a.g = ConvGeom{H, W, C, KW, SH, SW, DH, DW, OH, OW};
    return run_gemm<true>(a, vec, accumulate, workspace, workspace_bytes, s);
}
