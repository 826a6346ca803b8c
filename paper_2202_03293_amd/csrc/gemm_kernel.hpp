// The fp32 MFMA GEMM kernel template of liblg: matmul in its three operand layouts (Section 4.6.1,
// equations AB, A^T B, A B^T) and conv_2d_nhwc_hwcf (Section 4.6.2) as an implicit GEMM with
// M = N*OH*OW, N = F, K = KH*KW*C whose A operand is gathered from the NHWC input on the fly (the
// HWCF filter already is a row-major [K, F] matrix).
//
// Decomposition (the hardware counterpart of the paper's tile / pack / vectorise / contract steps):
//   grid      -> BM x BN output tiles, dealt so that each XCD's L2 sees a compact block of tiles
//   workgroup -> stages A and B k-slices (BK deep) global -> LDS directly (no registers), a ring of
//                three or four LDS stages with the transfers running two or three slices ahead of
//                the multiply
//   wavefront -> WM x WN register tile of 32x32 fp32 accumulators, v_mfma_f32_32x32x2_f32
//   epilogue  -> accumulators (+ C) straight to global memory
//   PERSIST   -> a grid smaller than the tile count: each workgroup walks over several tiles and starts the
//                transfers of its next tile before (or while) it finishes the current one, so that the
//                output stores drain under the next tile's multiplications (short contractions with a
//                large output, where writing C costs as much as computing it; AB and A^T B)
//
// An operand slice comes in one of two kinds, by which of its two axes is contiguous in memory:
//   R-kind (k contiguous: A of AB and A B^T, B of A B^T): LDS holds [rows][BK], the float4 column
//       XOR-swizzled with row bits; a lane reads FOUR consecutive k of its row with one
//       ds_read_b128 and feeds them to four MFMAs.  This works because the sum over k is order-free:
//       half-wave h of MFMA step 4j+i multiplies k = 8j + 4h + i, for both operands.
//   C-kind (m or n contiguous: B of AB and A^T B, A of A^T B): LDS holds [BK][cols] as in memory; a
//       lane reads one k-row per MFMA step.  For B the columns are interleaved over the accumulator
//       blocks (block nb holds columns NB*c + nb, c = lane % 32), so one ds_read_b{32*NB} feeds all
//       NB blocks and the epilogue finds NB adjacent columns of a row in one lane (128-bit stores).
#pragma once
#include "lg_common.hpp"
#include "gemm_plan.hpp"
#include <type_traits>

namespace lg {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// BM x BN output tile per workgroup, BK-deep k-slices, WM x WN register tile per wavefront.
// MINW = wavefronts per SIMD the register allocation must leave room for (what LDS lets a CU hold).
template <int BM_, int BN_, int BK_, int WM_, int WN_, int MINW_, int STAGES_ = 3, bool KTAIL_ = true>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MINW = MINW_;
    static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
    static constexpr int WAVES = WAVES_M * WAVES_N;
    static constexpr int THREADS = WAVES * kWave;
    static constexpr int MB = WM / 32;              // accumulator blocks along m per wave
    static constexpr int NB = WN / 32;              // along n (1, 2 or 4)
    static constexpr int QPR = BK / 4;              // float4s per row of an R-kind slice
    static constexpr int A_PER_T = BM * BK / 4 / THREADS;   // float4s of a slice per lane
    static constexpr int B_PER_T = BK * BN / 4 / THREADS;
    static constexpr int ROW_STEP = THREADS / QPR;  // R-kind: rows between a lane's successive float4s
    // LDS ring.  3: one slice being multiplied, two in flight.  4: three in flight and the barrier
    // publishes slices one step early, so a wave fetches the first fragments of the next slice
    // while it still multiplies the current one (see the main loop).
    static constexpr int STAGES = STAGES_;
    // Whether a k tail (slab depth not a multiple of BK) may follow the transfer ring as one
    // register-staged slice, or sends the whole tile down the register-staged path.  The big tile
    // opts out: the state the tail keeps alive across the ring does not fit its register budget.
    static constexpr bool KTAIL = KTAIL_;
    static_assert(STAGES == 3 || STAGES == 4, "ring depth");
    static constexpr int LDS_FLOATS = STAGES * (BM * BK + BK * BN);
    static_assert(BK == 16 || BK == 32 || BK == 64, "k-slice depth");
    static_assert(NB == 1 || NB == 2 || NB == 4, "wave tile width must be 32, 64 or 128");
    static_assert((BM * BK / 4) % THREADS == 0 && (BK * BN / 4) % THREADS == 0, "slice must divide over the workgroup");
    static_assert(THREADS % QPR == 0 && ROW_STEP % 16 == 0 && (THREADS / BK) % 8 == 0,
                  "a lane's R-kind rows must share one swizzle");

    // R-kind LDS position (in floats) of the float4 holding k = 4q .. 4q+3 of row r.  Rows are BK
    // floats; the quad index is XOR-ed with row bits so that the rows a read touches together land on
    // distinct banks.  The LDS of this part serves a 128-bit read 16 lanes at a time over 64 banks
    // (SQ_LDS_BANK_CONFLICT: with the row bits chosen for 8 lanes over 32 banks, rows 8 apart collided --
    // 17-50 % of the LDS cycles of every R-kind operand; with the bits below: 0).  16 consecutive rows
    // reading the same logical quad must therefore hit 16 distinct 4-bank groups: a row of BK = 16 floats
    // spans a quarter of the banks, so rows r, r+4, r+8, r+12 need four different quads (row bits 2-3);
    // a row of 32 floats spans half, so rows of equal parity need eight (row bits 1-3).
    // The one-float transfer path (VEC = false) keeps the narrower choice (bits 1-2 / 0-2): its rows per
    // lane are only 8 apart for BK = 32 and must share one swizzle; it is bound by its transfers anyway.
    template <bool VEC> static constexpr int swz_sh() { return VEC ? ((QPR == 4) ? 2 : (QPR == 8) ? 1 : 0) : ((QPR == 4) ? 1 : 0); }
    static constexpr int SWZ_MASK = (QPR < 8) ? QPR - 1 : 7;
    template <bool VEC> __device__ static __forceinline__ int swizzle(int r) { return (r >> swz_sh<VEC>()) & SWZ_MASK; }
    template <bool VEC> __device__ static __forceinline__ int r_off(int r, int q) { return r * BK + ((q ^ swizzle<VEC>(r)) << 2); }
};

template <class T, bool VEC, bool CONV, bool TA, bool TB, bool PERSIST = false>
__global__ __launch_bounds__(T::THREADS, T::MINW) void gemm_kernel(const GemmArgs p) {
    static_assert(!(CONV && (TA || TB)) && !(TA && TB), "supported operand layouts");
    static_assert(!PERSIST || (VEC && !CONV && !TB), "tile loop: aligned AB and A^T B only");
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, MB = T::MB, NB = T::NB, NTH = T::THREADS;
    constexpr int APT = T::A_PER_T, BPT = T::B_PER_T;
    extern __shared__ __align__(16) float lds[];
    float* As = lds;                               // [STAGES][BM*BK]
    float* Bs = lds + T::STAGES * BM * BK;         // [STAGES][BK*BN]

    // ---- which tile ------------------------------------------------------------------------
    const unsigned ntiles = p.tiles_m * p.tiles_n;
    constexpr unsigned GM = 8;     // tile rows per panel: the ~64 workgroups an XCD runs at once form an 8 x 8 block of tiles
    // Tile number v (a workgroup id, or with PERSIST one of blockIdx.x + i * gridDim.x: the grid is a multiple
    // of the XCD count, so all of a workgroup's tiles belong to its XCD's range) -> tile origin and the
    // rows / columns of the tile inside the matrix.
    int64_t m0, n0, m_valid, n_valid;
    auto place_tile = [&](unsigned v) {
        const unsigned L = xcd_contiguous_id(v, ntiles);
        const unsigned panel = L / (GM * p.tiles_n);
        const unsigned first_m = panel * GM;
        const unsigned gsz = (p.tiles_m - first_m < GM) ? p.tiles_m - first_m : GM;
        const unsigned in_panel = L - panel * GM * p.tiles_n;
        m0 = (int64_t)(first_m + in_panel % gsz) * BM;
        n0 = (int64_t)(in_panel / gsz) * BN;
        m_valid = (p.M - m0 < BM) ? p.M - m0 : BM;
        n_valid = (p.N - n0 < BN) ? p.N - n0 : BN;
    };
    unsigned vtile = blockIdx.x;
    place_tile(vtile);
    const int64_t kbeg = (int64_t)blockIdx.y * p.k_per_split;
    const int64_t kend = (kbeg + p.k_per_split < p.K) ? kbeg + p.k_per_split : p.K;
    const int nslices = (int)((kend - kbeg + BK - 1) / BK);

    const int t = threadIdx.x;
    const int lane = t % kWave, wave = t / kWave;
    const int wm0 = (wave / T::WAVES_N) * T::WM;   // wave tile origin inside the block tile
    const int wn0 = (wave % T::WAVES_N) * T::WN;
    const int c32 = lane % 32, h = lane / 32;

    // ---- staging coordinates ----------------------------------------------------------------------
    // Float4 number q = t + i*NTH of a slice is staged by lane t (its i-th float4) and lives at LDS
    // float offset 4q of the stage, for both kinds.  R-kind: q -> row q / QPR, physical quad q % QPR,
    // and the lane fetches the LOGICAL quad lq = physical ^ swizzle(row) (the same for all i), so the
    // swizzle costs nothing.  C-kind: q -> k-row q / (cols/4), column quad q % (cols/4).
    const int r0 = t / T::QPR;
    const int lq = (t % T::QPR) ^ T::template swizzle<VEC>(r0);

    // conv: element offset of GEMM row m = (n, oh, ow) at filter tap (0, 0), channel 0; grows with m
    // (M, OH, OW < 2^31 -- the host checks -- so the divisions are 32-bit: several times cheaper)
    auto conv_row_base = [&](int64_t m) -> int64_t {
        const uint32_t mu = (uint32_t)m, OWu = (uint32_t)p.g.OW, OHu = (uint32_t)p.g.OH;
        const uint32_t q = mu / OWu;
        const int64_t ow = mu - q * OWu, n = q / OHu, oh = q - (uint32_t)n * OHu;
        return ((n * p.g.H + oh * p.g.SH) * p.g.W + ow * p.g.SW) * p.g.C;
    };
    // R-kind row bases (element offset of the row's k = 0; -1 when the row is outside the matrix)
    int64_t a_rowbase[TA ? 1 : APT];
    int64_t b_rowbase[TB ? BPT : 1];
    auto row_bases = [&]() {
        if constexpr (!TA) {
#pragma unroll
            for (int i = 0; i < APT; ++i) {
                const int64_t m = m0 + r0 + i * T::ROW_STEP;
                if (m >= p.M) { a_rowbase[i] = -1; continue; }
                if constexpr (CONV) {
                    a_rowbase[i] = conv_row_base(m);
                } else {
                    a_rowbase[i] = m * p.lda;
                }
            }
        }
        if constexpr (TB) {
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                const int64_t n = n0 + r0 + i * T::ROW_STEP;
                b_rowbase[i] = n < p.N ? n * p.ldb : -1;
            }
        }
    };
    row_bases();
    float4 ra[APT], rb[BPT];

    auto conv_koff = [&](int64_t k) -> int64_t {   // conv: offset of GEMM column k relative to the row base
        const int64_t c = k % p.g.C, kk = k / p.g.C;
        const int64_t kw = kk % p.g.KW, kh = kk / p.g.KW;
        return (kh * p.g.DH * p.g.W + kw * p.g.DW) * p.g.C + c;
    };

    // ---- general (edge) slice loads: every access predicated ----------------------------------------
    auto load_R = [&](const float* base, const int64_t* rowbase, bool is_conv, int64_t k0, float4* regs, auto per_c) {
        constexpr int PER = decltype(per_c)::value;
        if constexpr (VEC) {
            const int64_t k = k0 + 4 * lq;
            const bool kin = k < kend;             // K % 4 == 0 on this path: a quad is all in or all out
            const int64_t ko = !kin ? 0 : (is_conv ? conv_koff(k) : k);
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                regs[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (kin && rowbase[i] >= 0) regs[i] = *reinterpret_cast<const float4*>(base + rowbase[i] + ko);
            }
        } else {
            int64_t ko[4];
            bool kin[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t k = k0 + 4 * lq + e;
                kin[e] = k < kend;
                ko[e] = !kin[e] ? 0 : (is_conv ? conv_koff(k) : k);
            }
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                if (rowbase[i] >= 0) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (kin[e]) v[e] = base[rowbase[i] + ko[e]];
                }
                regs[i] = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    };
    auto load_C = [&](const float* base, int64_t ld, int64_t col0, int64_t ncols, int64_t k0, float4* regs,
                      auto per_c, auto cols_c) {
        constexpr int PER = decltype(per_c)::value, CQ = decltype(cols_c)::value / 4;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int q = t + i * NTH;
            const int64_t k = k0 + q / CQ, c = col0 + 4 * (q % CQ);
            regs[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k < kend) {
                const float* ptr = base + k * ld + c;
                if constexpr (VEC) {
                    if (c < ncols) regs[i] = *reinterpret_cast<const float4*>(ptr);   // ncols % 4 == 0 here
                } else {
                    if (c + 0 < ncols) regs[i].x = ptr[0];
                    if (c + 1 < ncols) regs[i].y = ptr[1];
                    if (c + 2 < ncols) regs[i].z = ptr[2];
                    if (c + 3 < ncols) regs[i].w = ptr[3];
                }
            }
        }
    };
    auto load_slice_edge = [&](int64_t k0) {
        if constexpr (TA) load_C(p.A, p.lda, m0, p.M, k0, ra, std::integral_constant<int, APT>{}, std::integral_constant<int, BM>{});
        else              load_R(p.A, a_rowbase, CONV, k0, ra, std::integral_constant<int, APT>{});
        if constexpr (TB) load_R(p.B, b_rowbase, false, k0, rb, std::integral_constant<int, BPT>{});
        else              load_C(p.B, p.ldb, n0, p.N, k0, rb, std::integral_constant<int, BPT>{}, std::integral_constant<int, BN>{});
    };
    auto store_slice = [&](int buf) {
        float* as = As + buf * (BM * BK);
        float* bs = Bs + buf * (BK * BN);
#pragma unroll
        for (int i = 0; i < APT; ++i) *reinterpret_cast<float4*>(as + 4 * (t + i * NTH)) = ra[i];
#pragma unroll
        for (int i = 0; i < BPT; ++i) *reinterpret_cast<float4*>(bs + 4 * (t + i * NTH)) = rb[i];
    };

    // ---- interior slices: global -> LDS transfers ---------------------------------------------------
    // Whole tile inside M x N, whole slices inside the k-slab, aligned operands.  global_load_lds_dwordx4
    // moves 16 bytes per lane straight into LDS, the 64 lanes of a wave filling 1 KiB at consecutive
    // addresses, which is exactly the lane-order layout above.  Addresses are a wave-uniform base
    // (advanced by scalar adds) plus a per-lane 32-bit byte offset that never changes, so the main
    // loop spends no vector ALU instruction on addressing (vector ALU instructions are not free
    // here: they take issue slots from the matrix pipe, which small tiles feel).
    const char* a_base = reinterpret_cast<const char*>(p.A);
    const char* b_base = reinterpret_cast<const char*>(p.B);
    // transfers per lane per slice: one per float4 of the slice (aligned operands), one per float otherwise
    constexpr int APD = VEC ? APT : 4 * APT, BPD = VEC ? BPT : 4 * BPT;
    uint32_t a_loff[APD], b_loff[BPD];
    int64_t a_adv = 0, b_adv = 0;                  // bytes per k-slice
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);

    // Convolution gather: a quad sits at filter tap (kh, kw), channel c; its byte offset from the row
    // base advances by BK channels per slice, and when c passes C the tap moves on (kw, then kh),
    // which changes the offset by constants.  When C is a multiple of BK a slice never straddles a
    // tap, the walk is the same for all lanes and lives in scalar registers (su_*); otherwise each
    // lane walks its own quad (cv_*), branch-free when C >= BK.
    const int cvC = (int)p.g.C, cvKW = (int)p.g.KW;
    const uint32_t cv_d_kw = (uint32_t)((p.g.DW * p.g.C - p.g.C) * 4);                          // c wraps, kw + 1
    const uint32_t cv_d_kh = (uint32_t)((p.g.DH * p.g.W * p.g.C - p.g.KW * p.g.DW * p.g.C) * 4);  // kw wraps, kh + 1
    const bool conv_uniform = CONV && (cvC % BK == 0);
    int cv_c = 0, cv_kw = 0, cv_kh = 0, su_c = 0, su_kw = 0;
    uint32_t cv_off = 0, su_off = 0;
    auto cv_offset = [&]() {
        return (uint32_t)((((int64_t)cv_kh * p.g.DH * p.g.W + (int64_t)cv_kw * p.g.DW) * p.g.C + cv_c) * 4);
    };

    // Tiles on the M or N boundary use the transfers too: a lane whose row or column lies outside the
    // matrix fetches the last valid row / column quad instead (in bounds, and what it feeds are
    // accumulators the epilogue never stores).  `valid` = rows (columns) of the tile inside the matrix.
    auto r_loff = [&](int64_t ld, uint32_t* loff, int64_t valid, auto per_c) {   // R-kind lane offsets from (row0, kbeg)
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < decltype(per_c)::value; ++i) {
                int64_t r = r0 + i * T::ROW_STEP;
                if (r >= valid) r = valid - 1;
                loff[i] = (uint32_t)((r * ld + 4 * lq) * 4);
            }
        } else {
            // float number f = t + i*NTH of the slice sits at LDS float offset f: row f / BK, physical
            // quad (f % BK) / 4, element f % 4 -- the lane fetches the logical quad's element
#pragma unroll
            for (int i = 0; i < 4 * decltype(per_c)::value; ++i) {
                const int f = t + i * NTH;
                int64_t r = f / BK;
                const int kq = (((f % BK) / 4) ^ T::template swizzle<VEC>((int)r)) * 4 + f % 4;
                if (r >= valid) r = valid - 1;
                loff[i] = (uint32_t)((r * ld + kq) * 4);
            }
        }
    };
    auto c_loff = [&](int64_t ld, uint32_t* loff, int64_t valid, auto per_c, auto cols_c) {   // C-kind, from (kbeg, col0)
        if constexpr (VEC) {
            constexpr int CQ = decltype(cols_c)::value / 4;
#pragma unroll
            for (int i = 0; i < decltype(per_c)::value; ++i) {
                const int q = t + i * NTH;
                int64_t c = 4 * (q % CQ);
                if (c >= valid) c = valid - 4;         // valid is a multiple of 4 on this path
                loff[i] = (uint32_t)(((int64_t)(q / CQ) * ld + c) * 4);
            }
        } else {
            constexpr int COLS = decltype(cols_c)::value;
#pragma unroll
            for (int i = 0; i < 4 * decltype(per_c)::value; ++i) {
                const int f = t + i * NTH;
                int64_t c = f % COLS;
                if (c >= valid) c = valid - 1;
                loff[i] = (uint32_t)(((int64_t)(f / COLS) * ld + c) * 4);
            }
        }
    };
    auto init_full = [&]() {
        a_base = reinterpret_cast<const char*>(p.A);
        b_base = reinterpret_cast<const char*>(p.B);
        if constexpr (CONV) {
            // lane offsets are relative to the tile's first row, so only the tile has to span < 2 GiB
            const int64_t base0 = to_scalar(conv_row_base(m0));
            a_base += base0 * 4;
            auto conv_base_clamped = [&](int i) -> int64_t {   // row base of the lane's i-th row, or of row M-1
                return a_rowbase[TA ? 0 : i] >= 0 ? a_rowbase[TA ? 0 : i] : conv_row_base(p.M - 1);
            };
            // The lane's k position inside a slice is the same for all its transfers: the logical quad
            // lq (aligned operands), or -- one float per transfer -- element t % 4 of the logical quad at
            // physical position t % BK (the rows of a lane's transfers are NTH / BK apart, which leaves
            // the swizzle unchanged).
            const int row_t = t / BK;
            const int lk = VEC ? 4 * lq : (((t % BK) / 4) ^ T::template swizzle<VEC>(row_t)) * 4 + t % 4;
            auto lane_row_base = [&](int i) -> int64_t {
                if constexpr (VEC) {
                    return conv_base_clamped(i);
                } else {
                    const int64_t m = m0 + row_t + i * (NTH / BK);
                    return conv_row_base(m < p.M ? m : p.M - 1);
                }
            };
            if (conv_uniform) {
                su_c = (int)(kbeg % p.g.C);
                su_kw = (int)((kbeg / p.g.C) % p.g.KW);
                const int64_t kh = kbeg / (p.g.C * p.g.KW);
                su_off = (uint32_t)(((kh * p.g.DH * p.g.W + (int64_t)su_kw * p.g.DW) * p.g.C + su_c) * 4);
#pragma unroll
                for (int i = 0; i < APD; ++i) a_loff[i] = (uint32_t)((lane_row_base(i) - base0 + lk) * 4);
            } else {
                const int64_t k = kbeg + lk;
                cv_c = (int)(k % p.g.C);
                cv_kw = (int)((k / p.g.C) % p.g.KW);
                cv_kh = (int)(k / (p.g.C * p.g.KW));
                cv_off = cv_offset();
#pragma unroll
                for (int i = 0; i < APD; ++i) a_loff[i] = (uint32_t)((lane_row_base(i) - base0) * 4);
            }
        } else if constexpr (TA) {
            a_base += (kbeg * p.lda + m0) * 4;
            a_adv = (int64_t)BK * p.lda * 4;
            c_loff(p.lda, a_loff, m_valid, std::integral_constant<int, APT>{}, std::integral_constant<int, BM>{});
        } else {
            a_base += (m0 * p.lda + kbeg) * 4;
            a_adv = BK * 4;
            r_loff(p.lda, a_loff, m_valid, std::integral_constant<int, APT>{});
        }
        if constexpr (TB) {
            b_base += (n0 * p.ldb + kbeg) * 4;
            b_adv = BK * 4;
            r_loff(p.ldb, b_loff, n_valid, std::integral_constant<int, BPT>{});
        } else {
            b_base += (kbeg * p.ldb + n0) * 4;
            b_adv = (int64_t)BK * p.ldb * 4;
            c_loff(p.ldb, b_loff, n_valid, std::integral_constant<int, BPT>{}, std::integral_constant<int, BN>{});
        }
        // the transfer instruction takes its base from scalar registers: pin both there once, so that
        // the per-slice advances below are scalar adds whatever else uses the operand pointers
        a_base = reinterpret_cast<const char*>(to_scalar(reinterpret_cast<int64_t>(a_base)));
        b_base = reinterpret_cast<const char*>(to_scalar(reinterpret_cast<int64_t>(b_base)));
    };
    // Start the transfer of the next slice into LDS stage `buf`.
    auto issue_slice = [&](int buf) {
        constexpr int WORDS = VEC ? 4 : 1;         // floats per lane per transfer
        float* as = As + buf * (BM * BK) + WORDS * 64 * wave_u;
        float* bs = Bs + buf * (BK * BN) + WORDS * 64 * wave_u;
        auto dma = [&](const void* base, uint32_t voff, uint32_t lds_a) __attribute__((always_inline)) {
            if constexpr (VEC) dma16(base, voff, lds_a); else dma4(base, voff, lds_a);
        };
        // (in the tile loop the bases are carried from tile to tile: say again that they are uniform)
        const char* a_sb = PERSIST ? reinterpret_cast<const char*>(to_scalar(reinterpret_cast<int64_t>(a_base))) : a_base;
        const char* b_sb = PERSIST ? reinterpret_cast<const char*>(to_scalar(reinterpret_cast<int64_t>(b_base))) : b_base;
        if (CONV && conv_uniform) {
            const char* ab = a_sb + su_off;
#pragma unroll
            for (int i = 0; i < APD; ++i) dma(ab, a_loff[i], lds_addr(as + WORDS * i * NTH));
        } else {
            const uint32_t ko = CONV ? cv_off : 0u;
#pragma unroll
            for (int i = 0; i < APD; ++i) dma(a_sb, a_loff[i] + ko, lds_addr(as + WORDS * i * NTH));
        }
#pragma unroll
        for (int i = 0; i < BPD; ++i) dma(b_sb, b_loff[i], lds_addr(bs + WORDS * i * NTH));
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
            a_base += a_adv;
        }
        b_base += b_adv;
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
    // Software-pipelined: R-kind fragments (4 k per read) are fetched up front, the C-kind fragment of
    // step st+1 is fetched before the MFMAs of step st are issued, so LDS latency hides behind
    // MB*NB*64 cycles of matrix work instead of stalling the in-order wave.
    auto compute_slice = [&](int buf) {
        const float* as = As + buf * (BM * BK);
        const float* bs = Bs + buf * (BK * BN);
        constexpr int NJ = BK / 8, NSTEP = BK / 2;
        float4 a4[TA ? 1 : NJ][MB];
        float4 b4[TB ? NJ : 1][NB];
        float a1[2][MB], b1[2][NB];
        if constexpr (!TA) {
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    a4[j][mb] = *reinterpret_cast<const float4*>(as + T::template r_off<VEC>(wm0 + mb * 32 + c32, 2 * j + h));
        }
        if constexpr (TB) {      // block nb holds columns nb*32 + c32: consecutive lanes read consecutive rows
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    b4[j][nb] = *reinterpret_cast<const float4*>(bs + T::template r_off<VEC>(wn0 + nb * 32 + c32, 2 * j + h));
        }
        auto load_step = [&](int st, int slot) {
            const int k = 8 * (st / 4) + 4 * h + (st % 4);
            if constexpr (TA) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) a1[slot][mb] = as[k * BM + wm0 + mb * 32 + c32];
            }
            if constexpr (!TB) {
                const float* brow = bs + k * BN + wn0 + NB * c32;
                if constexpr (NB == 4) {
                    const float4 v = *reinterpret_cast<const float4*>(brow);
                    b1[slot][0] = v.x; b1[slot][1] = v.y; b1[slot][2] = v.z; b1[slot][3] = v.w;
                } else if constexpr (NB == 2) {
                    const float2 v = *reinterpret_cast<const float2*>(brow);
                    b1[slot][0] = v.x; b1[slot][1] = v.y;
                } else {
                    b1[slot][0] = *brow;
                }
            }
        };
        auto comp = [](const float4& v, int i) { return (i == 0) ? v.x : (i == 1) ? v.y : (i == 2) ? v.z : v.w; };
        load_step(0, 0);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            if (st + 1 < NSTEP) load_step(st + 1, (st + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
            const int j = st / 4, i = st % 4;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                float av;
                if constexpr (TA) av = a1[st & 1][mb]; else av = comp(a4[j][mb], i);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    float bv;
                    if constexpr (TB) bv = comp(b4[j][nb], i); else bv = b1[st & 1][nb];
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[mb][nb], 0, 0, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // The same, for the ring of four stages: the slice after this one is already visible in LDS, so
    // its R-kind fragments (register set `1 - set`) and its first C-kind step are fetched while this
    // slice is multiplied; on entry this slice's own (set `set`, step 0 in slot 0) are in registers.
    // A wave then crosses the barrier between slices with its next operands in hand, instead of
    // starting the LDS reads after it.
    constexpr int NJ = BK / 8, NSTEP = BK / 2;
    float4 pa4[2][TA ? 1 : NJ][MB];
    float4 pb4[2][TB ? NJ : 1][NB];
    float pa1[2][MB], pb1[2][NB];
    auto fetch_R = [&](int buf, int set) {
        const float* as = As + buf * (BM * BK);
        const float* bs = Bs + buf * (BK * BN);
        if constexpr (!TA) {
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    pa4[set][j][mb] = *reinterpret_cast<const float4*>(as + T::template r_off<VEC>(wm0 + mb * 32 + c32, 2 * j + h));
        }
        if constexpr (TB) {
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    pb4[set][j][nb] = *reinterpret_cast<const float4*>(bs + T::template r_off<VEC>(wn0 + nb * 32 + c32, 2 * j + h));
        }
    };
    auto fetch_C = [&](int buf, int st, int slot) {
        const float* as = As + buf * (BM * BK);
        const float* bs = Bs + buf * (BK * BN);
        const int k = 8 * (st / 4) + 4 * h + (st % 4);
        if constexpr (TA) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) pa1[slot][mb] = as[k * BM + wm0 + mb * 32 + c32];
        }
        if constexpr (!TB) {
            const float* brow = bs + k * BN + wn0 + NB * c32;
            if constexpr (NB == 4) {
                const float4 v = *reinterpret_cast<const float4*>(brow);
                pb1[slot][0] = v.x; pb1[slot][1] = v.y; pb1[slot][2] = v.z; pb1[slot][3] = v.w;
            } else if constexpr (NB == 2) {
                const float2 v = *reinterpret_cast<const float2*>(brow);
                pb1[slot][0] = v.x; pb1[slot][1] = v.y;
            } else {
                pb1[slot][0] = *brow;
            }
        }
    };
    auto compute_slice_ahead = [&](int buf, int nextbuf, int set) {
        auto comp = [](const float4& v, int i) { return (i == 0) ? v.x : (i == 1) ? v.y : (i == 2) ? v.z : v.w; };
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            if (st + 1 < NSTEP) fetch_C(buf, st + 1, (st + 1) & 1);
            else                fetch_C(nextbuf, 0, 0);          // NSTEP is even: slot 0 is free again
            if (st == 1) fetch_R(nextbuf, 1 - set);
            __builtin_amdgcn_sched_barrier(0);
            const int j = st / 4, i = st % 4;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                float av;
                if constexpr (TA) av = pa1[st & 1][mb]; else av = comp(pa4[set][j][mb], i);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    float bv;
                    if constexpr (TB) bv = comp(pb4[set][j][nb], i); else bv = pb1[st & 1][nb];
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[mb][nb], 0, 0, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop --------------------------------------------------------------------------
    // The interior path addresses operands with 32-bit byte offsets from the tile origin.
    const int64_t lim = (int64_t)1 << 31;
    const bool b_small = (int64_t)(TB ? BN : BK) * p.ldb * 4 < lim;
    // All tiles (boundary tiles included, see r_loff) run their whole slices through the transfer rings
    // below -- 16 bytes per lane for aligned operands, 4 otherwise -- and a k tail (a slab whose depth
    // is not a multiple of BK) as one last predicated, register-staged slice.  Left to the
    // register-staged path: spans beyond 32-bit offsets.
    bool interior, ktail;
    int nring;
    auto classify = [&]() {
        bool a_small;
        if constexpr (CONV) {      // rows of the tile x the filter's reach, from the tile's first row
            const int64_t last = (m0 + BM <= p.M) ? m0 + BM - 1 : p.M - 1;
            const int64_t kh_taps = p.K / (p.g.KW * p.g.C);
            const int64_t reach = ((kh_taps - 1) * p.g.DH * p.g.W + (p.g.KW - 1) * p.g.DW + 1) * p.g.C;
            a_small = (conv_row_base(last) - conv_row_base(m0) + reach + BK) * 4 < lim;
        } else {
            a_small = (int64_t)(TA ? BK : BM) * p.lda * 4 < lim;
        }
        // (the flag is wave-uniform; readfirstlane says so to the compiler where 32-bit divisions left it
        // in vector registers, so that the branches below stay scalar)
        interior = __builtin_amdgcn_readfirstlane(
            (int)(a_small && b_small && (T::KTAIL || (kend - kbeg) % BK == 0))) != 0;
        nring = interior ? (int)((kend - kbeg) / BK) : 0;
        ktail = T::KTAIL && interior && (kend - kbeg) % BK != 0;
    };
    classify();
    constexpr int LT = APD + BPD;              // transfers per slice per wave
    // The first slices of a tile: as many as the ring keeps in flight, into stages 0, 1, (2).
    auto prologue = [&]() {
        init_full();
        issue_slice(0);
        if (nring > 1) issue_slice(1);
        if (T::STAGES == 4 && nring > 2) issue_slice(2);
    };

    // The tile loop (PERSIST; without it the body runs once).  What it is for: a wave's stores and
    // transfers complete in the order issued, so a wait for a transfer also waits for every store issued
    // before it.  The next tile's first transfers are therefore issued BEFORE this tile's stores, and
    // the waits that follow name the stores in their counts, so that the stores drain while the next
    // tile is multiplied.  Those counts must be exact: they are only used after an epilogue that issued
    // exactly NST stores per lane (the whole tile inside C, nothing to accumulate, nothing predicated).
    // Two forms:
    //   continuous -- four-stage ring, slices per tile a multiple of four (so every tile starts at stage 0):
    //       the ring runs on across tiles; the last three steps of a tile issue the next tile's slices
    //       0 .. 2, and the wave arrives at the next tile with that tile's first fragments in registers;
    //   ahead      -- otherwise: after the last step the next tile's prologue is issued, then the stores.
    constexpr bool kCanOverlap = PERSIST && VEC && !TB && (NB == 4 || NB == 2);
    constexpr int NST = MB * 16;               // stores per lane of an unpredicated epilogue
    static_assert(!kCanOverlap || LT + NST <= 63, "the wait counter holds 63");
    bool ahead = false;        // this tile's prologue was issued before the last tile's NST stores
    bool cont = false;         // continuous form: this tile's slices 0 .. 2 are issued, its first fragments fetched
    bool counted = false;      // ... and exactly NST stores of the last tile follow slice 2 in issue order
    for (;;) {
        const unsigned vnext = vtile + gridDim.x;
        const bool has_next = PERSIST && vnext < ntiles;
        const int64_t em0 = m0, en0 = n0;              // the epilogue's tile (the transfers may move on before it)
        const bool whole = m_valid == BM && n_valid == BN && !p.accumulate;
        // (a k tail is staged through stage 0 after the ring: the ring must not have moved on by then)
        const bool continuous = kCanOverlap && T::STAGES == 4 && nring >= 4 && nring % 4 == 0 && !ktail;
        if (continuous) {
            if (!cont) {
                prologue();
                dma_wait<LT>();
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                fetch_R(0, 0);
                fetch_C(0, 0, 0);
            }
            auto step = [&](auto stage_c, int s) {
                constexpr int stage = decltype(stage_c)::value;
                if (s + 3 == nring && has_next) {      // from here on the transfers belong to the next tile
                    place_tile(vnext);
                    init_full();
                }
                const bool issued = s + 3 < nring || has_next;
                if (issued) issue_slice((stage + 3) % 4);
                compute_slice_ahead(stage, (stage + 1) % 4, stage & 1);
                if (s + 2 < nring || has_next) {
                    if (!issued) dma_wait<0>();
                    else if (s == 0 && counted) dma_wait<LT + NST>();   // slice 2, the last tile's stores, slice 3
                    else dma_wait<LT>();
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
            };
            for (int s = 0; s < nring; s += 4) {
                step(std::integral_constant<int, 0>{}, s);
                step(std::integral_constant<int, 1>{}, s + 1);
                step(std::integral_constant<int, 2>{}, s + 2);
                step(std::integral_constant<int, 3>{}, s + 3);
            }
        } else if (nring > 0 && T::STAGES == 4) {
            // Ring of four LDS stages, transfers three slices ahead.  The barrier that ends step s makes
            // slice s+2 visible (each wave first waits for its own transfers of that slice), so during
            // step s+1 every wave may already read slice s+2.  It also guarantees that nobody still
            // reads slice s, whose stage the transfer issued in step s+1 refills.
            if (!ahead) {
                prologue();
                if (nring > 2) dma_wait<LT>(); else dma_wait<0>();
            } else {                                   // slices 0, 1, (2), then NST stores; 0 and 1 are needed
                if (nring > 2) dma_wait<LT + NST>(); else dma_wait<NST>();
            }
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            fetch_R(0, 0);
            fetch_C(0, 0, 0);
            auto step = [&](auto stage_c, int s) {
                constexpr int stage = decltype(stage_c)::value;
                if (s + 3 < nring) issue_slice((stage + 3) % 4);
                compute_slice_ahead(stage, (stage + 1) % 4, stage & 1);
                if (s + 2 < nring) {
                    if (s + 3 < nring) dma_wait<LT>(); else dma_wait<0>();
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
            };
            int s = 0;
            for (; s + 4 <= nring; s += 4) {
                step(std::integral_constant<int, 0>{}, s);
                step(std::integral_constant<int, 1>{}, s + 1);
                step(std::integral_constant<int, 2>{}, s + 2);
                step(std::integral_constant<int, 3>{}, s + 3);
            }
            if (s < nring) step(std::integral_constant<int, 0>{}, s);
            if (s + 1 < nring) step(std::integral_constant<int, 1>{}, s + 1);
            if (s + 2 < nring) step(std::integral_constant<int, 2>{}, s + 2);
        } else if (nring > 0) {
            // Ring of three LDS stages, transfers two slices ahead.  Each wave waits for its own
            // transfers of the slice needed next (vmcnt counts them in order), then the barrier makes
            // everybody's visible and also guarantees nobody still reads the stage refilled next.
            if (!ahead) {
                prologue();
                if (nring > 1) dma_wait<LT>(); else dma_wait<0>();
            } else {                                   // slices 0, (1), then NST stores; 0 is needed
                if (nring > 1) dma_wait<LT + NST>(); else dma_wait<NST>();
            }
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // One trip = three slices, one per LDS stage, so that every LDS address in the loop is a
            // lane constant plus an immediate (no vector ALU work per slice).
            auto step = [&](auto stage_c, int s) {
                constexpr int stage = decltype(stage_c)::value;
                if (s + 2 < nring) issue_slice((stage + 2) % 3);
                compute_slice(stage);
                if (s + 1 < nring) {
                    if (s + 2 < nring) dma_wait<LT>(); else dma_wait<0>();
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
            };
            int s = 0;
            for (; s + 3 <= nring; s += 3) {
                step(std::integral_constant<int, 0>{}, s);
                step(std::integral_constant<int, 1>{}, s + 1);
                step(std::integral_constant<int, 2>{}, s + 2);
            }
            if (s < nring) step(std::integral_constant<int, 0>{}, s);
            if (s + 1 < nring) step(std::integral_constant<int, 1>{}, s + 1);
        } else if (!interior && nslices > 0) {
            // Registers -> LDS, two of the ring's stages.
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
        if (ktail) {
            if (nring > 0) __syncthreads();        // every wave is done with the ring's stages
            load_slice_edge(kbeg + (int64_t)nring * BK);
            store_slice(0);
            __syncthreads();
            compute_slice(0);
        }

        // ---- the workgroup's next tile ------------------------------------------------------------
        ahead = false;
        cont = false;
        counted = false;
        if constexpr (PERSIST) {
            if (continuous && has_next) {          // already placed, its slices 0 .. 2 on their way
                cont = true;
                counted = whole;
            } else if (has_next) {
                __syncthreads();                   // every wave is done reading the ring's stages
                place_tile(vnext);
                row_bases();
                classify();
                if (kCanOverlap && whole && nring > 0) {   // (not continuous: every tile has this tile's nring)
                    prologue();
                    ahead = true;
                }
            }
            vtile = vnext;
        }
        const bool unpredicated = cont ? counted : ahead;

        // ---- epilogue ------------------------------------------------------------------------------
        // accumulator register r of block (mb, nb): row = 32*mb + 8*(r/4) + 4*h + r%4;
        // column = NB*c32 + nb (interleaved, C-kind B) or nb*32 + c32 (R-kind B)
        float* Cz = p.C + (int64_t)blockIdx.y * p.M * p.ldc;
        if constexpr (!VEC && !TB && NB > 1) {
            // An output that cannot take 128-bit stores: written straight from the accumulators, the lanes
            // of a store would sit NB columns apart (1/NB-dense instructions).  Each wavefront instead
            // turns one 32 x WN block at a time around in its own piece of LDS (the ring is done) and
            // writes whole rows: 64 adjacent floats per store instruction.
            constexpr int WN = T::WN;
            static_assert(T::WAVES * 32 * WN <= T::LDS_FLOATS, "the staging blocks must fit the ring's LDS");
            __syncthreads();                               // every wave is done reading the ring's stages
            float* ws = lds + wave * (32 * WN);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float* q = ws + (8 * (r / 4) + 4 * h + (r % 4)) * WN + NB * c32;
                    if constexpr (NB == 4) *reinterpret_cast<float4*>(q) = make_float4(acc[mb][0][r], acc[mb][1][r], acc[mb][2][r], acc[mb][3][r]);
                    else                   *reinterpret_cast<float2*>(q) = make_float2(acc[mb][0][r], acc[mb][1][r]);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < 32 * WN / kWave; ++it) {
                    const int idx = it * kWave + lane;
                    const int64_t m = em0 + wm0 + mb * 32 + idx / WN;
                    const int64_t n = en0 + wn0 + idx % WN;
                    const float v = ws[idx];
                    if (m < p.M && n < p.N) {
                        float* cp = Cz + m * p.ldc + n;
                        *cp = p.accumulate ? *cp + v : v;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        } else if (kCanOverlap && unpredicated) {
            // the whole tile, overwritten: exactly NST store instructions per lane (the waits above count them)
            if constexpr (kCanOverlap) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int64_t m = em0 + wm0 + mb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                        float* cp = Cz + m * p.ldc + en0 + wn0 + NB * c32;
                        if constexpr (NB == 4)
                            __builtin_nontemporal_store(f32x4{acc[mb][0][r], acc[mb][1][r], acc[mb][2][r], acc[mb][3][r]},
                                                        reinterpret_cast<f32x4*>(cp));
                        else
                            __builtin_nontemporal_store(f32x2{acc[mb][0][r], acc[mb][1][r]}, reinterpret_cast<f32x2*>(cp));
                    }
                }
            }
        } else {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t m = em0 + wm0 + mb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                    if (m >= p.M) continue;
                    float v[NB];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) v[nb] = acc[mb][nb][r];
                    if constexpr (TB) {
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            const int64_t n = en0 + wn0 + nb * 32 + c32;
                            float* cp = Cz + m * p.ldc + n;
                            if (n < p.N) *cp = p.accumulate ? *cp + v[nb] : v[nb];
                        }
                    } else {
                        const int64_t ncol = en0 + wn0 + NB * c32;
                        float* cp = Cz + m * p.ldc + ncol;
                        if constexpr (VEC && NB == 4) {
                            if (ncol < p.N) {
                                float4 o = make_float4(v[0], v[1], v[2], v[3]);
                                if (p.accumulate) {
                                    const float4 c = *reinterpret_cast<const float4*>(cp);
                                    o.x += c.x; o.y += c.y; o.z += c.z; o.w += c.w;
                                }
                                // written once, never read back here: stream it past the caches that hold A and B
                                __builtin_nontemporal_store(f32x4{o.x, o.y, o.z, o.w}, reinterpret_cast<f32x4*>(cp));
                            }
                        } else if constexpr (VEC && NB == 2) {
                            if (ncol < p.N) {
                                float2 o = make_float2(v[0], v[1]);
                                if (p.accumulate) {
                                    const float2 c = *reinterpret_cast<const float2*>(cp);
                                    o.x += c.x; o.y += c.y;
                                }
                                __builtin_nontemporal_store(f32x2{o.x, o.y}, reinterpret_cast<f32x2*>(cp));
                            }
                        } else {
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb)
                                if (ncol + nb < p.N) cp[nb] = p.accumulate ? cp[nb] + v[nb] : v[nb];
                        }
                    }
                }
            }
        }
        if (!has_next) break;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;
    }
}


// ---- the tile menu ----------------------------------------------------------------------------------
// All tiles: 4 wavefronts, one per SIMD.  The big tile keeps three LDS stages: a fourth would cost it
// its second workgroup per CU.  The host-side table of these tiles (same order) and the planner
// that picks among them are in gemm_plan.hpp.
using Tile0 = Tile<128, 256, 16, 64, 128, 2, 3, false>;   // waves of 64x128
using Tile1 = Tile<128, 128, 16, 32, 128, 2, 4>;   // waves of 32x128
using Tile2 = Tile<128, 64, 16, 32, 64, 3, 4>;     // waves of 32x64 (narrow outputs, e.g. F = 64)
using Tile3 = Tile<64, 64, 16, 32, 32, 4, 4>;      // waves of 32x32 (small problems)
using Tile4 = Tile<64, 128, 32, 32, 64, 2>;        // waves of 32x64, deeper slices (mid-size problems)
using Tile5 = Tile<64, 64, 32, 32, 32, 2, 4>;      // waves of 32x32, deeper slices
using Tile6 = Tile<128, 32, 32, 32, 32, 2, 3>;     // four waves of 32x32 stacked along m: tall products with few columns
using Tile7 = Tile<32, 128, 32, 32, 32, 2, 3>;     // four waves of 32x32 side by side: a few rows times a large matrix

// The tiles compiled with the tile loop as well (aligned AB and A^T B: the layouts whose epilogue writes
// 64- or 128-bit rows): see make_plan for when it is used.
template <class T> constexpr bool kHasTileLoop = std::is_same_v<T, Tile1> || std::is_same_v<T, Tile2> || std::is_same_v<T, Tile4>;

// `persist_grid` > 0: that many workgroups (a multiple of the XCD count, fewer than there are tiles) walk
// over the tiles, where the tile loop is compiled; one workgroup per tile otherwise.
template <class T, bool VEC, bool CONV, bool TA, bool TB>
static void launch_gemm(const GemmArgs& a, unsigned splits, unsigned persist_grid, hipStream_t s) {
    const size_t lds_bytes = T::LDS_FLOATS * sizeof(float);
    const unsigned ntiles = a.tiles_m * a.tiles_n;
    if constexpr (VEC && !CONV && !TB && kHasTileLoop<T>) {
        const unsigned grid = persist_grid / kXcds * kXcds;
        if (grid > 0 && grid < ntiles && splits == 1) {
            static DeviceFlags configured_loop = {};
            allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_kernel<T, VEC, CONV, TA, TB, true>), lds_bytes, configured_loop);
            hipLaunchKernelGGL((gemm_kernel<T, VEC, CONV, TA, TB, true>), dim3(grid, 1), dim3(T::THREADS), lds_bytes, s, a);
            return;
        }
    }
    static DeviceFlags configured = {};
    allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_kernel<T, VEC, CONV, TA, TB>), lds_bytes, configured);
    hipLaunchKernelGGL((gemm_kernel<T, VEC, CONV, TA, TB>), dim3(ntiles, splits), dim3(T::THREADS), lds_bytes, s, a);
}

// Launch the planned tile of one operand-layout variant (the split-k combine is the caller's job).
template <bool CONV, bool TA, bool TB>
static void launch_planned(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s) {
    const unsigned z = (unsigned)pl.splits, pg = (unsigned)pl.persist_grid;
#define LG_LAUNCH(TILE)                                                        \
    do {                                                                       \
        if (vec) launch_gemm<TILE, true, CONV, TA, TB>(a, z, pg, s);           \
        else     launch_gemm<TILE, false, CONV, TA, TB>(a, z, pg, s);          \
    } while (0)
    switch (pl.tile) {
        case 0: LG_LAUNCH(Tile0); break;
        case 1: LG_LAUNCH(Tile1); break;
        case 2: LG_LAUNCH(Tile2); break;
        case 3: LG_LAUNCH(Tile3); break;
        case 4: LG_LAUNCH(Tile4); break;
        case 5: LG_LAUNCH(Tile5); break;
        case 6: LG_LAUNCH(Tile6); break;
        default: LG_LAUNCH(Tile7); break;
    }
#undef LG_LAUNCH
}

// Implemented in gemm.hip (AB and convolution) and gemm_t.hip (A^T B, A B^T).
void launch_nn(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s);
void launch_conv(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s);
void launch_tn(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s);
void launch_nt(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s);

}  // namespace lg
