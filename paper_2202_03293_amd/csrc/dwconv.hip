// Depthwise convolutions (Section 4.7): no contraction across channels, so no matrix cores;
// K_w (or K_h*K_w) FMAs per output element against 8 bytes of traffic -> HBM-bound.
//
// 3x3 in 2-D at strides and dilations 1 and 2 with channel counts that are multiples of 32: output tiles
// whose input patch is staged in LDS by direct global->LDS transfers and consumed row by row while the
// rest is still in flight (dwconv2d_tile_kernel, dwconv2d_tile_sd_kernel).
// Register-window kernels (filter widths 3, 5, 7 in 1-D, 3x3 in 2-D; strides and dilations 1 and 2,
// the values the paper sweeps): a lane owns 4 adjacent channels (one 128-bit access) and a few output
// positions, keeps the input window in registers so each input element is loaded once per lane, and
// neighbouring lanes/workgroups share the halo through L2.  A row-streaming kernel covers the other
// filter widths up to 9 at horizontal stride and dilation 1 (5x5, 7x7); general kernels cover any
// other stride, dilation, filter size and channel count, one output position per lane.
#include "lg_common.hpp"

namespace lg {

constexpr int kDThreads = 256;
constexpr int kDw2RowGroup = 2;   // vertically adjacent patches of the 2-D window kernel that share a lane group
                                  // (measured 1, 2, 4: 2 is 3-7 % ahead at dilation 1, behind at dilation 2)

typedef float f32x4 __attribute__((ext_vector_type(4)));

// 128-bit streaming store: the output is written once and not read again by this kernel.
__device__ __forceinline__ void store_stream4(float* p, const float4 v) {
    __builtin_nontemporal_store(f32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4*>(p));
}

__device__ __forceinline__ float4 fma4(const float4 a, const float4 b, const float4 c) {
    return make_float4(fmaf(a.x, b.x, c.x), fmaf(a.y, b.y, c.y), fmaf(a.z, b.z, c.z), fmaf(a.w, b.w, c.w));
}

// ---- register-window kernels: compile-time filter size, stride and dilation ---------------------
// A lane owns T outputs along a dimension, G apart, where G = D / gcd(S, D) is the output spacing
// at which neighbouring outputs share input positions (1 except for dilation 2 at stride 1, where
// outputs of equal parity share).  Output j (at G*j from the lane's first) reads window positions
// j*G*S + i*D for taps i < K: only those positions are loaded, each once.
constexpr int gcd_i(int a, int b) { return b == 0 ? a : gcd_i(b, a % b); }

template <int K, int S, int D, int T>
struct Window {
    static constexpr int G = D / gcd_i(S, D);
    static constexpr int SPAN = (T - 1) * G * S + (K - 1) * D + 1;
    static constexpr bool used(int p) {
        for (int j = 0; j < T; ++j)
            for (int i = 0; i < K; ++i)
                if (j * G * S + i * D == p) return true;
        return false;
    }
    // last window position needed when only n of the T outputs exist
    __device__ static __forceinline__ int reach(int n) { return (n - 1) * G * S + (K - 1) * D; }
};

// 1-D, C % 4 == 0.  Lane -> (n, run of TW outputs, 4 channels); channels vary fastest across lanes
// so a wavefront reads 1 KiB contiguous per input position.  Runs are numbered (block, phase):
// block b, phase p holds outputs b*G*TW + p + G*j.
template <int KW, int SW, int DW, int TW>
__global__ __launch_bounds__(kDThreads) void dwconv1d_win_kernel(
    const float* __restrict__ I, const float* __restrict__ Kf, float* __restrict__ O,
    int64_t N, int64_t W, int64_t C, int64_t OW, int accumulate, unsigned nblocks) {
    using Win = Window<KW, SW, DW, TW>;
    constexpr int G = Win::G;
    const int64_t C4 = C / 4;
    const int64_t runs = (OW + G * TW - 1) / (G * TW) * G;
    const int64_t total = N * runs * C4;
    const int64_t idx = (int64_t)xcd_contiguous_id(blockIdx.x, nblocks) * kDThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t c4 = idx % C4;
    const int64_t run = (idx / C4) % runs;
    const int64_t n = idx / (C4 * runs);
    const int64_t w0 = (run / G) * (G * TW) + run % G;
    if (w0 >= OW) return;
    const int64_t left = (OW - w0 + G - 1) / G;
    const int nout = left < TW ? (int)left : TW;
    float4 k[KW];
#pragma unroll
    for (int i = 0; i < KW; ++i) k[i] = *reinterpret_cast<const float4*>(Kf + i * C + 4 * c4);
    const float* ip = I + (n * W + w0 * SW) * C + 4 * c4;
    float* op = O + (n * OW + w0) * C + 4 * c4;
    float4 x[Win::SPAN];
    const int reach = Win::reach(nout);
#pragma unroll
    for (int p = 0; p < Win::SPAN; ++p) {
        x[p] = make_float4(0, 0, 0, 0);
        if (Win::used(p) && p <= reach) x[p] = *reinterpret_cast<const float4*>(ip + (int64_t)p * C);
    }
#pragma unroll
    for (int j = 0; j < TW; ++j) {
        if (j < nout) {
            float* q = op + (int64_t)(G * j) * C;
            // the initial accumulator enters last so that overwrite and accumulate share the k-sum
            float4 s = make_float4(0, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < KW; ++i) s = fma4(x[j * G * SW + i * DW], k[i], s);
            if (accumulate) {
                const float4 acc = *reinterpret_cast<const float4*>(q);
                s.x += acc.x; s.y += acc.y; s.z += acc.z; s.w += acc.w;
            }
            *reinterpret_cast<float4*>(q) = s;
        }
    }
}

// 2-D, same stride S and dilation D in both dimensions, C % 4 == 0.  Lane -> (n, TH x TW outputs G
// apart, 4 channels).  The whole input patch is requested before any arithmetic, so a lane exposes
// one memory latency, not one per row (measured 27 -> 19 us on the 8x114x114x96 workload against a
// rolling row window).  Outputs are streamed with non-temporal stores.  Plain workgroup order:
// the XCD-contiguous order measured slightly slower here.
template <int KH, int KW, int S, int D, int TH, int TW>
__global__ __launch_bounds__(kDThreads) void dwconv2d_win_kernel(
    const float* __restrict__ I, const float* __restrict__ Kf, float* __restrict__ O,
    int64_t N, int64_t H, int64_t W, int64_t C, int64_t OH, int64_t OW, int accumulate, int RB) {
    using WinH = Window<KH, S, D, TH>;
    using WinW = Window<KW, S, D, TW>;
    constexpr int G = WinH::G;
    const int64_t C4 = C / 4;
    const int64_t pw = (OW + G * TW - 1) / (G * TW) * G, ph = (OH + G * TH - 1) / (G * TH) * G;
    // lane order: channels, then RB vertically adjacent patches (they share halo rows: same workgroup,
    // same L1), then patches along the row
    const int64_t phb = (ph + RB - 1) / RB;
    const int64_t total = N * phb * RB * pw * C4;
    const int64_t idx = (int64_t)blockIdx.x * kDThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t c4 = idx % C4;
    const int64_t q = idx / C4;                       // RB is 1 or a power of two: no division for it
    const int sh = RB > 1 ? 31 - __builtin_clz((unsigned)RB) : 0;
    const int64_t rb = q & (RB - 1), q2 = q >> sh;
    const int64_t bw = q2 % pw, q3 = q2 / pw;
    const int64_t bh = (q3 % phb) * RB + rb;
    const int64_t n = q3 / phb;
    if (bh >= ph) return;
    const int64_t h0 = (bh / G) * (G * TH) + bh % G, w0 = (bw / G) * (G * TW) + bw % G;
    if (h0 >= OH || w0 >= OW) return;
    const int64_t left_h = (OH - h0 + G - 1) / G, left_w = (OW - w0 + G - 1) / G;
    const int nh = left_h < TH ? (int)left_h : TH;
    const int nw = left_w < TW ? (int)left_w : TW;
    const float* ip = I + ((n * H + h0 * S) * W + w0 * S) * C + 4 * c4;
    float* op = O + ((n * OH + h0) * OW + w0) * C + 4 * c4;
    float4 x[WinH::SPAN][WinW::SPAN];
    const int reach_h = WinH::reach(nh), reach_w = WinW::reach(nw);
#pragma unroll
    for (int r = 0; r < WinH::SPAN; ++r)
#pragma unroll
        for (int c = 0; c < WinW::SPAN; ++c) {
            x[r][c] = make_float4(0, 0, 0, 0);
            if (WinH::used(r) && WinW::used(c) && r <= reach_h && c <= reach_w)
                x[r][c] = *reinterpret_cast<const float4*>(ip + ((int64_t)r * W + c) * C);
        }
    float4 k[KH][KW];
#pragma unroll
    for (int a = 0; a < KH; ++a)
#pragma unroll
        for (int b = 0; b < KW; ++b) k[a][b] = *reinterpret_cast<const float4*>(Kf + (a * KW + b) * C + 4 * c4);
#pragma unroll
    for (int r = 0; r < TH; ++r)
#pragma unroll
        for (int o = 0; o < TW; ++o) {
            if (r < nh && o < nw) {
                float4 s = make_float4(0, 0, 0, 0);
#pragma unroll
                for (int a = 0; a < KH; ++a)
#pragma unroll
                    for (int b = 0; b < KW; ++b) s = fma4(x[r * G * S + a * D][o * G * S + b * D], k[a][b], s);
                float* q = op + ((int64_t)(G * r) * OW + G * o) * C;
                if (accumulate) {
                    const float4 acc = *reinterpret_cast<const float4*>(q);
                    s.x += acc.x; s.y += acc.y; s.z += acc.z; s.w += acc.w;
                }
                store_stream4(q, s);
            }
        }
}

// 2-D, 3 x 3, stride 1, dilation 1, overwriting output, channels in slabs of CS4 quads: tiles through LDS.
//
// A workgroup owns TH x TW output pixels of one image for one slab of 4*CS4 channels.  The
// (TH+2) x (TW+2) input patch it needs -- and the nine filter taps of its channels -- are moved
// global -> LDS by the lanes' direct transfers (16 bytes each, no registers), all requested up front,
// so every input element crosses from L2 to the compute unit once per tile instead of once per tap row,
// and the halo between neighbouring tiles is re-read from the L2 they share (tiles are numbered so
// that an accelerator die works on one image at a time).  Lane -> (channel quad, column of the tile);
// it walks down the tile's rows with a 3-row window in registers and streams one output per row.
//
// The rows are consumed while the rest of the patch is still in flight.  On this architecture a
// wave's vector memory operations, loads and stores alike, share one counter and complete in issue
// order (the compiler's own s_waitcnt placement rests on the same property), so "input rows <= r
// have landed" is "at most (transfers of later rows + stores issued since) are outstanding": an
// s_waitcnt with a compile-time count per row, then a workgroup barrier (each wave has waited for its
// own transfers, the barrier publishes everybody's).  Leaving the stores out of the count -- waiting
// for them too -- is correct under any completion order and measured 1 us (6 %) slower.
// That count is exact only if every lane issues every store, so all tiles are full: tiles at the
// bottom and right edge are moved inwards and recompute a few outputs of their neighbours (the same
// values, bit for bit).  The host sends shapes smaller than a tile, and accumulating calls, elsewhere.
constexpr int ceil_div_i(int a, int b) { return (a + b - 1) / b; }
constexpr int min_i(int a, int b) { return a < b ? a : b; }

template <int CS4, int TH, int TW>
struct Dw2Tile {
    static constexpr int T = CS4 * TW;                        // lanes: one per (channel quad, column)
    static constexpr int THp = TH + 2, TWp = TW + 2;
    static constexpr int ROW = TWp * CS4;                     // 128-bit words per patch row
    static constexpr int ITEMS = THp * ROW;
    static constexpr int NL = ceil_div_i(ITEMS, T);           // transfers per lane for the patch
    static constexpr int KNL = ceil_div_i(9 * CS4, T);        // ... and for the filter
    static constexpr int LDS_BYTES = (KNL + NL) * T * 16;
    static_assert(T % kWave == 0 && T <= 1024, "whole wavefronts");
    static_assert(NL + TH <= 63, "the wait counts must fit s_waitcnt's 6 bits");
};

template <int CS4, int TH, int TW>
__global__ __launch_bounds__(CS4 * TW) void dwconv2d_tile_kernel(
    const float* __restrict__ I, const float* __restrict__ Kf, float* __restrict__ O,
    int64_t H, int64_t W, int64_t C, int64_t OH, int64_t OW,
    unsigned ntiles, unsigned tiles_h, unsigned tiles_w, unsigned slabs) {
    using D = Dw2Tile<CS4, TH, TW>;
    constexpr int T = D::T, TWp = D::TWp, ROW = D::ROW, ITEMS = D::ITEMS, NL = D::NL, KNL = D::KNL;
    extern __shared__ __align__(16) float4 dw_lds[];          // [KNL*T] filter taps, then [NL*T] patch
    float4* kf = dw_lds;
    float4* patch = dw_lds + KNL * T;
    const unsigned L = xcd_contiguous_id(blockIdx.x, ntiles);
    const unsigned slab = L % slabs, tw = (L / slabs) % tiles_w;
    const unsigned th = (L / (slabs * tiles_w)) % tiles_h, n = L / (slabs * tiles_w * tiles_h);
    int64_t h0 = (int64_t)th * TH, w0 = (int64_t)tw * TW;
    if (h0 > OH - TH) h0 = OH - TH;                           // edge tiles move inwards: every tile is full
    if (w0 > OW - TW) w0 = OW - TW;
    const int t = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(t / kWave);
    {
        const char* kb = reinterpret_cast<const char*>(to_scalar(reinterpret_cast<int64_t>(Kf + slab * CS4 * 4)));
#pragma unroll
        for (int i = 0; i < KNL; ++i) {
            int q = i * T + t;
            if (q > 9 * CS4 - 1) q = 9 * CS4 - 1;             // spare lanes repeat the last word (LDS has room for them)
            const int tap = q / CS4, c4 = q - tap * CS4;
            dma16(kb, (uint32_t)((tap * C + 4 * c4) * 4), lds_addr(kf + i * T + wave * kWave));
        }
    }
    const char* base = reinterpret_cast<const char*>(
        to_scalar(reinterpret_cast<int64_t>(I + ((n * H + h0) * W + w0) * C + slab * CS4 * 4)));
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        int q = i * T + t;
        if (q > ITEMS - 1) q = ITEMS - 1;
        const int r = q / ROW, rem = q - r * ROW;
        const int px = rem / CS4, c4 = rem - px * CS4;
        dma16(base, (uint32_t)(((r * W + px) * C + 4 * c4) * 4), lds_addr(patch + i * T + wave * kWave));
    }
    const int c4 = t % CS4, col = t / CS4;
    float* op = O + ((n * OH + h0) * OW + w0 + col) * C + slab * CS4 * 4 + 4 * c4;
    float4 k[3][3];
    float4 x[3][3];
    static_for<0, TH + 2>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        constexpr int last = min_i(ceil_div_i((r + 1) * ROW, T) - 1, NL - 1);   // last transfer that brings a word of row r
        constexpr int stores = r >= 2 ? r - 2 : 0;                               // issued by every lane so far
        dma_wait<min_i(NL - 1 - last + stores, 63)>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if constexpr (r == 0) {
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b) k[a][b] = kf[(a * 3 + b) * CS4 + c4];
        }
#pragma unroll
        for (int b = 0; b < 3; ++b) x[r % 3][b] = patch[(r * TWp + col + b) * CS4 + c4];
        if constexpr (r >= 2) {
            constexpr int oh = r - 2;
            float4 s = make_float4(0, 0, 0, 0);
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b) s = fma4(x[(oh + a) % 3][b], k[a][b], s);
            store_stream4(op + (int64_t)oh * OW * C, s);
        }
    });
}

// The same staging at the other strides and dilations the paper sweeps (S, D in {1, 2}, equal in both
// dimensions).  Only input positions that some (output, tap) pair reads are staged: they lie g = gcd(S, D)
// apart, so patch position (pr, pc) is input position (h0*S + g*pr, w0*S + g*pc) and output (oh, ow) reads
// patch rows oh*S/g + a*D/g, columns ow*S/g + b*D/g -- which is also the paper's byte accounting (input
// bytes divided by the product of the gcds).  The nine taps are read from LDS per output (no register
// window: at stride 2 neighbouring output rows share one input row at most).
template <int CS4, int TH, int TW, int S, int D>
struct Dw2TileSD {
    static constexpr int G = gcd_i(S, D), SG = S / G, DG = D / G;
    static constexpr int T = CS4 * TW;
    static constexpr int PR = (TH - 1) * SG + 2 * DG + 1, PC = (TW - 1) * SG + 2 * DG + 1;
    static constexpr int ROW = PC * CS4, ITEMS = PR * ROW;
    static constexpr int NL = ceil_div_i(ITEMS, T), KNL = ceil_div_i(9 * CS4, T);
    static constexpr int LDS_BYTES = (KNL + NL) * T * 16;
    static_assert(T % kWave == 0 && T <= 1024, "whole wavefronts");
    static_assert(NL + TH <= 63, "the wait counts must fit s_waitcnt's 6 bits");
    static_assert(LDS_BYTES <= 160 * 1024, "tile must fit in LDS");
};

template <int CS4, int TH, int TW, int S, int D>
__global__ __launch_bounds__(CS4 * TW) void dwconv2d_tile_sd_kernel(
    const float* __restrict__ I, const float* __restrict__ Kf, float* __restrict__ O,
    int64_t H, int64_t W, int64_t C, int64_t OH, int64_t OW,
    unsigned ntiles, unsigned tiles_h, unsigned tiles_w, unsigned slabs) {
    using Dd = Dw2TileSD<CS4, TH, TW, S, D>;
    constexpr int T = Dd::T, PC = Dd::PC, ROW = Dd::ROW, ITEMS = Dd::ITEMS, NL = Dd::NL, KNL = Dd::KNL;
    constexpr int G = Dd::G, SG = Dd::SG, DG = Dd::DG;
    extern __shared__ __align__(16) float4 dw_lds[];          // [KNL*T] filter taps, then [NL*T] patch
    float4* kf = dw_lds;
    float4* patch = dw_lds + KNL * T;
    const unsigned L = xcd_contiguous_id(blockIdx.x, ntiles);
    const unsigned slab = L % slabs, tw = (L / slabs) % tiles_w;
    const unsigned th = (L / (slabs * tiles_w)) % tiles_h, n = L / (slabs * tiles_w * tiles_h);
    int64_t h0 = (int64_t)th * TH, w0 = (int64_t)tw * TW;
    if (h0 > OH - TH) h0 = OH - TH;                           // edge tiles move inwards: every tile is full
    if (w0 > OW - TW) w0 = OW - TW;
    const int t = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(t / kWave);
    {
        const char* kb = reinterpret_cast<const char*>(to_scalar(reinterpret_cast<int64_t>(Kf + slab * CS4 * 4)));
#pragma unroll
        for (int i = 0; i < KNL; ++i) {
            int q = i * T + t;
            if (q > 9 * CS4 - 1) q = 9 * CS4 - 1;
            const int tap = q / CS4, c4 = q - tap * CS4;
            dma16(kb, (uint32_t)((tap * C + 4 * c4) * 4), lds_addr(kf + i * T + wave * kWave));
        }
    }
    const char* base = reinterpret_cast<const char*>(
        to_scalar(reinterpret_cast<int64_t>(I + ((n * H + h0 * S) * W + w0 * S) * C + slab * CS4 * 4)));
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        int q = i * T + t;
        if (q > ITEMS - 1) q = ITEMS - 1;
        const int r = q / ROW, rem = q - r * ROW;
        const int px = rem / CS4, c4 = rem - px * CS4;
        dma16(base, (uint32_t)(((r * G * W + px * G) * C + 4 * c4) * 4), lds_addr(patch + i * T + wave * kWave));
    }
    const int c4 = t % CS4, col = t / CS4;
    float* op = O + ((n * OH + h0) * OW + w0 + col) * C + slab * CS4 * 4 + 4 * c4;
    float4 k[3][3];
    static_for<0, TH>([&](auto ohc) {
        constexpr int oh = decltype(ohc)::value;
        constexpr int need = oh * SG + 2 * DG;                                     // last patch row this output row reads
        constexpr int last = min_i(ceil_div_i((need + 1) * ROW, T) - 1, NL - 1);   // last transfer that brings a word of it
        dma_wait<min_i(NL - 1 - last + oh, 63)>();                                 // + the oh stores every lane has issued
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if constexpr (oh == 0) {
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b) k[a][b] = kf[(a * 3 + b) * CS4 + c4];
        }
        float4 s = make_float4(0, 0, 0, 0);
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
            for (int b = 0; b < 3; ++b)
                s = fma4(patch[((oh * SG + a * DG) * PC + col * SG + b * DG) * CS4 + c4], k[a][b], s);
        store_stream4(op + (int64_t)oh * OW * C, s);
    });
}

template <int CS4, int TH, int TW, int S, int D>
static int launch_dw2_tile_sd(const float* I, const float* Kf, float* O, int64_t N, int64_t H, int64_t W, int64_t C,
                              int64_t OH, int64_t OW, hipStream_t s) {
    using Dd = Dw2TileSD<CS4, TH, TW, S, D>;
    const int64_t tiles_h = cdiv(OH, TH), tiles_w = cdiv(OW, TW), slabs = C / (4 * CS4);
    const int64_t ntiles = N * tiles_h * tiles_w * slabs;
    if (ntiles > kMaxGrid) return LG_ERR_UNSUPPORTED;
    static DeviceFlags configured = {};
    allow_dynamic_lds(reinterpret_cast<const void*>(&dwconv2d_tile_sd_kernel<CS4, TH, TW, S, D>), Dd::LDS_BYTES, configured);
    hipLaunchKernelGGL((dwconv2d_tile_sd_kernel<CS4, TH, TW, S, D>), dim3((unsigned)ntiles), dim3(Dd::T), Dd::LDS_BYTES, s,
                       I, Kf, O, H, W, C, OH, OW, (unsigned)ntiles, (unsigned)tiles_h, (unsigned)tiles_w, (unsigned)slabs);
    return launch_status();
}

template <int CS4, int TH, int TW, int S, int D>
static bool dw2_tile_sd_fits(int64_t W, int64_t C, int64_t OH, int64_t OW) {
    using Dd = Dw2TileSD<CS4, TH, TW, S, D>;
    return C % (4 * CS4) == 0 && OH >= TH && OW >= TW && (int64_t)Dd::PR * Dd::G * W * C * 4 < ((int64_t)1 << 31);
}

template <int CS4, int TH, int TW>
static int launch_dw2_tile(const float* I, const float* Kf, float* O, int64_t N, int64_t H, int64_t W, int64_t C,
                           int64_t OH, int64_t OW, hipStream_t s) {
    using D = Dw2Tile<CS4, TH, TW>;
    const int64_t tiles_h = cdiv(OH, TH), tiles_w = cdiv(OW, TW), slabs = C / (4 * CS4);
    const int64_t ntiles = N * tiles_h * tiles_w * slabs;
    if (ntiles > kMaxGrid) return LG_ERR_UNSUPPORTED;
    static DeviceFlags configured = {};
    allow_dynamic_lds(reinterpret_cast<const void*>(&dwconv2d_tile_kernel<CS4, TH, TW>), D::LDS_BYTES, configured);
    hipLaunchKernelGGL((dwconv2d_tile_kernel<CS4, TH, TW>), dim3((unsigned)ntiles), dim3(D::T), D::LDS_BYTES, s,
                       I, Kf, O, H, W, C, OH, OW, (unsigned)ntiles, (unsigned)tiles_h, (unsigned)tiles_w, (unsigned)slabs);
    return launch_status();
}

// what the tile kernel takes: whole tiles, channel slabs, lane offsets inside a patch within 32 bits
template <int CS4, int TH, int TW>
static bool dw2_tile_fits(int64_t W, int64_t C, int64_t OH, int64_t OW) {
    return C % (4 * CS4) == 0 && OH >= TH && OW >= TW && (TH + 2) * W * C * 4 < ((int64_t)1 << 31);
}

// Row-streaming kernel for the filters the window kernels do not cover (5x5, 7x7, 1-D widths
// 2 ... 9): horizontal stride and dilation 1, C % 4 == 0, any filter height, vertical stride and
// dilation.  A lane owns a run of TW outputs of one output row for 4 channels and walks the filter
// rows: per filter row it loads the TW + KW - 1 input positions its run touches and the KW taps,
// then does TW * KW multiply-adds -- (TW + 2*KW - 1) / TW loads per output and filter row instead of
// the 2*KW of one output per lane.  Vertical reuse (neighbouring output rows read the same input
// rows) is left to the caches.
// V = 4: a lane owns 4 adjacent channels (128-bit accesses; C % 4 == 0, 16-byte aligned tensors);
// V = 1: one channel per lane, for channel counts and alignments that rule those out.
// window position c is read by some (output o < T, tap b < K) of a run of consecutive outputs
template <int K, int S, int D, int T>
constexpr bool rows_used(int c) {
    for (int o = 0; o < T; ++o)
        for (int b = 0; b < K; ++b)
            if (o * S + b * D == c) return true;
    return false;
}

template <int V> struct ChanVec;
template <> struct ChanVec<4> {
    float4 v;
    __device__ static __forceinline__ ChanVec zero() { return {make_float4(0, 0, 0, 0)}; }
    __device__ static __forceinline__ ChanVec load(const float* p) { return {*reinterpret_cast<const float4*>(p)}; }
    __device__ __forceinline__ void fma(const ChanVec& a, const ChanVec& b) { v = fma4(a.v, b.v, v); }
    __device__ __forceinline__ void add(const ChanVec& a) { v.x += a.v.x; v.y += a.v.y; v.z += a.v.z; v.w += a.v.w; }
    __device__ __forceinline__ void store(float* p) const { store_stream4(p, v); }
};
template <> struct ChanVec<1> {
    float v;
    __device__ static __forceinline__ ChanVec zero() { return {0.f}; }
    __device__ static __forceinline__ ChanVec load(const float* p) { return {*p}; }
    __device__ __forceinline__ void fma(const ChanVec& a, const ChanVec& b) { v = fmaf(a.v, b.v, v); }
    __device__ __forceinline__ void add(const ChanVec& a) { v += a.v; }
    __device__ __forceinline__ void store(float* p) const { __builtin_nontemporal_store(v, p); }
};

// SW, DW: horizontal stride and dilation (1 or 2): the run's outputs then read window positions
// o*SW + b*DW, and only those are loaded (for stride 2 a run of 4 outputs of a 5-wide filter loads
// 11 positions and 5 taps instead of the 40 loads of four single outputs).
template <int KW, int TW, int V, int SW = 1, int DW = 1>
__global__ __launch_bounds__(kDThreads) void dwconv_rows_kernel(
    const float* __restrict__ I, const float* __restrict__ Kf, float* __restrict__ O,
    int64_t N, int64_t H, int64_t W, int64_t C, int64_t KH, int64_t SH, int64_t DH,
    int64_t OH, int64_t OW, int accumulate, int RB) {
    using CV = ChanVec<V>;
    // Lane order: channel group fastest, then RB vertically adjacent output rows, then the run along
    // the row, then blocks of RB rows, then the image: the lanes of a workgroup that read the same
    // input rows (neighbouring output rows) sit together and meet in L1.
    const int64_t CG = C / V, runs = (OW + TW - 1) / TW;       // channel groups of V
    const int64_t OHB = (OH + RB - 1) / RB;
    const int64_t total = N * OHB * runs * RB * CG;
    const int64_t idx = (int64_t)blockIdx.x * kDThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t cg = idx % CG;
    const int64_t q = idx / CG;                       // RB is 1 or a power of two: no division for it
    const int sh = RB > 1 ? 31 - __builtin_clz((unsigned)RB) : 0;
    const int64_t r = q & (RB - 1), q2 = q >> sh;
    const int64_t run = q2 % runs, q3 = q2 / runs;
    const int64_t ohb = q3 % OHB;
    const int64_t n = q3 / OHB;
    const int64_t oh = ohb * RB + r;
    if (oh >= OH) return;
    const int64_t w0 = run * TW;
    const int nw = OW - w0 < TW ? (int)(OW - w0) : TW;
    constexpr int SPAN = (TW - 1) * SW + (KW - 1) * DW + 1;
    const float* ip = I + ((n * H + oh * SH) * W + w0 * SW) * C + V * cg;
    const int reach = (nw - 1) * SW + (KW - 1) * DW;   // last window position the run's nw outputs read
    CV acc[TW];
#pragma unroll
    for (int o = 0; o < TW; ++o) acc[o] = CV::zero();
    for (int64_t a = 0; a < KH; ++a) {
        const float* row = ip + a * DH * W * C;
        CV x[SPAN], k[KW];
#pragma unroll
        for (int c = 0; c < SPAN; ++c) {
            x[c] = CV::zero();
            if (rows_used<KW, SW, DW, TW>(c) && c <= reach) x[c] = CV::load(row + (int64_t)c * C);
        }
#pragma unroll
        for (int b = 0; b < KW; ++b) k[b] = CV::load(Kf + (a * KW + b) * C + V * cg);
#pragma unroll
        for (int o = 0; o < TW; ++o)
#pragma unroll
            for (int b = 0; b < KW; ++b) acc[o].fma(x[o * SW + b * DW], k[b]);
    }
    float* op = O + ((n * OH + oh) * OW + w0) * C + V * cg;
#pragma unroll
    for (int o = 0; o < TW; ++o) {
        if (o < nw) {
            float* q = op + (int64_t)o * C;
            CV s = acc[o];
            if (accumulate) s.add(CV::load(q));
            s.store(q);
        }
    }
}

// General depthwise kernel (1-D is H = KH = 1): one output element per lane, channels fastest.
__global__ __launch_bounds__(kDThreads) void dwconv_general_kernel(
    const float* __restrict__ I, const float* __restrict__ Kf, float* __restrict__ O,
    int64_t N, int64_t H, int64_t W, int64_t C, int64_t KH, int64_t KW,
    int64_t SH, int64_t SW, int64_t DH, int64_t DW, int64_t OH, int64_t OW, int accumulate) {
    const int64_t total = N * OH * OW * C;
    const int64_t idx = (int64_t)blockIdx.x * kDThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t c = idx % C;
    const int64_t w = (idx / C) % OW;
    const int64_t h = (idx / (C * OW)) % OH;
    const int64_t n = idx / (C * OW * OH);
    float s = 0.f;
    for (int64_t a = 0; a < KH; ++a)
        for (int64_t b = 0; b < KW; ++b)
            s = fmaf(I[((n * H + h * SH + a * DH) * W + w * SW + b * DW) * C + c], Kf[(a * KW + b) * C + c], s);
    if (accumulate) s += O[idx];
    O[idx] = s;
}

// General depthwise kernel for C % 4 == 0: one output position x 4 channels per lane, any filter
// size, stride and dilation (the paper sweeps strides and dilations 1 and 2, Section 4.7).  Taps
// are read through L1/L2; neighbouring lanes share them.
__global__ __launch_bounds__(kDThreads) void dwconv_general_vec4_kernel(
    const float* __restrict__ I, const float* __restrict__ Kf, float* __restrict__ O,
    int64_t N, int64_t H, int64_t W, int64_t C, int64_t KH, int64_t KW,
    int64_t SH, int64_t SW, int64_t DH, int64_t DW, int64_t OH, int64_t OW, int accumulate) {
    const int64_t C4 = C / 4;
    const int64_t total = N * OH * OW * C4;
    const int64_t idx = (int64_t)blockIdx.x * kDThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t c4 = idx % C4;
    const int64_t w = (idx / C4) % OW;
    const int64_t h = (idx / (C4 * OW)) % OH;
    const int64_t n = idx / (C4 * OW * OH);
    const float* ip = I + ((n * H + h * SH) * W + w * SW) * C + 4 * c4;
    const float* kp = Kf + 4 * c4;
    float4 s = make_float4(0, 0, 0, 0);
    for (int64_t a = 0; a < KH; ++a)
        for (int64_t b = 0; b < KW; ++b)
            s = fma4(*reinterpret_cast<const float4*>(ip + (a * DH * W + b * DW) * C),
                     *reinterpret_cast<const float4*>(kp + (a * KW + b) * C), s);
    float* q = O + 4 * idx;
    if (accumulate) {
        const float4 acc = *reinterpret_cast<const float4*>(q);
        s.x += acc.x; s.y += acc.y; s.z += acc.z; s.w += acc.w;
    }
    store_stream4(q, s);
}

static int dwconv_dispatch(const float* I, const float* Kf, float* O,
                           int64_t N, int64_t H, int64_t W, int64_t C, int64_t KH, int64_t KW,
                           int64_t SH, int64_t SW, int64_t DH, int64_t DW, int accumulate, void* stream) {
    if (N < 0 || H < 0 || W < 0 || C < 0 || KH < 1 || KW < 1) return LG_ERR_INVALID_ARG;
    if (SH < 1 || SW < 1 || DH < 1 || DW < 1) return LG_ERR_INVALID_ARG;
    if (N == 0 || C == 0) return LG_OK;
    const int64_t OH = lg_conv_out_extent(H, KH, SH, DH), OW = lg_conv_out_extent(W, KW, SW, DW);
    if (OH == 0 || OW == 0) return LG_ERR_INVALID_ARG;
    if (!I || !Kf || !O) return LG_ERR_INVALID_ARG;
    const int64_t in_elems = N * H * W * C, out_elems = N * OH * OW * C;
    if (overlaps(I, in_elems * 4, O, out_elems * 4) || overlaps(Kf, KH * KW * C * 4, O, out_elems * 4))
        return LG_ERR_INVALID_ARG;
    hipStream_t s = begin_call(stream);
    const bool vec = (C % 4 == 0) && aligned16(I) && aligned16(Kf) && aligned16(O);
    const bool sd12 = SW >= 1 && SW <= 2 && DW >= 1 && DW <= 2;
    if (vec && KH == 1 && SH == 1 && DH == 1 && sd12 && (KW == 3 || KW == 5 || KW == 7)) {
        constexpr int TW = 4;    // measured best: short runs, many lanes in flight
        // H rows of a 1-D problem are independent images: fold them into N
        const int64_t NN = N * H;
        const int64_t G = DW / (SW == DW ? DW : 1);            // D / gcd(S, D) for S, D in {1, 2}
        const int64_t items = NN * (cdiv(OW, G * TW) * G) * (C / 4);
        const int64_t blocks = cdiv(items, kDThreads);
        if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
#define LG_DW1(K_, S_, D_)                                                                                   \
        if (KW == K_ && SW == S_ && DW == D_) {                                                              \
            hipLaunchKernelGGL((dwconv1d_win_kernel<K_, S_, D_, TW>), dim3((unsigned)blocks), dim3(kDThreads), \
                               0, s, I, Kf, O, NN, W, C, OW, accumulate, (unsigned)blocks);                  \
            return launch_status();                                                                          \
        }
        LG_DW1(3, 1, 1) LG_DW1(3, 2, 1) LG_DW1(3, 1, 2) LG_DW1(3, 2, 2)
        LG_DW1(5, 1, 1) LG_DW1(5, 2, 1) LG_DW1(5, 1, 2) LG_DW1(5, 2, 2)
        LG_DW1(7, 1, 1) LG_DW1(7, 2, 1) LG_DW1(7, 1, 2) LG_DW1(7, 2, 2)
#undef LG_DW1
    }
    // 3 x 3 at stride and dilation 1, overwriting: 8 x 16 pixel tiles x 32 channels through LDS (measured on
    // 8 x 114 x 114 x 96, cold: 20.7 -> 17.3 us back to back, input fetched from memory 1.47 -> 1.00 times)
    if (vec && KH == 3 && KW == 3 && SH == 1 && SW == 1 && DH == 1 && DW == 1 && !accumulate &&
        dw2_tile_fits<8, 8, 16>(W, C, OH, OW))
        return launch_dw2_tile<8, 8, 16>(I, Kf, O, N, H, W, C, OH, OW, s);
    // ... and at the other strides and dilations of the sweep, unless the tiles moved inwards at the edges would
    // recompute more than a quarter of the outputs (measured, cold: 32 x 114 x 114 x 96 dilation 2 68.6 -> 57.9 us,
    // stride 2 40.7 -> 39.5, both 20.1 -> 19.3; 32 x 58 x 58 x 256 stride and dilation 2, 27 x 27 outputs in
    // 8 x 16 tiles, 14.3 -> 15.4: left to the register-window kernel)
    if (vec && KH == 3 && KW == 3 && SH == SW && DH == DW && sd12 && !accumulate) {
#define LG_DW2SD(S_, D_, TH_)                                                                                \
        if (SW == S_ && DW == D_ && dw2_tile_sd_fits<8, TH_, 16, S_, D_>(W, C, OH, OW) &&                    \
            4 * cdiv(OH, TH_) * TH_ * cdiv(OW, 16) * 16 <= 5 * OH * OW)                                      \
            return launch_dw2_tile_sd<8, TH_, 16, S_, D_>(I, Kf, O, N, H, W, C, OH, OW, s);
        LG_DW2SD(2, 1, 4) LG_DW2SD(1, 2, 8) LG_DW2SD(2, 2, 8)
#undef LG_DW2SD
    }
    if (vec && KH == 3 && KW == 3 && SH == SW && DH == DW && sd12) {
        const int64_t G = DW / (SW == DW ? DW : 1);
#define LG_DW2(S_, D_, TH_, TW_)                                                                             \
        if (SW == S_ && DW == D_) {                                                                          \
            const int64_t ph_ = cdiv(OH, G * TH_) * G;                                                       \
            const int RB = (D_ == 1 && ph_ >= kDw2RowGroup) ? kDw2RowGroup : 1;                              \
            const int64_t items = N * (cdiv(ph_, RB) * RB) * (cdiv(OW, G * TW_) * G) * (C / 4);              \
            const int64_t blocks = cdiv(items, kDThreads);                                                   \
            if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;                                                \
            hipLaunchKernelGGL((dwconv2d_win_kernel<3, 3, S_, D_, TH_, TW_>), dim3((unsigned)blocks),        \
                               dim3(kDThreads), 0, s, I, Kf, O, N, H, W, C, OH, OW, accumulate, RB);         \
            return launch_status();                                                                          \
        }
        // patch sizes: small enough that the problem fills 256 CUs and the patch fits in registers
        LG_DW2(1, 1, 4, 2) LG_DW2(2, 1, 2, 2) LG_DW2(1, 2, 4, 2) LG_DW2(2, 2, 4, 2)
#undef LG_DW2
    }
    // (with few channels a wavefront's lanes would sit a whole run of pixels apart: left to the general
    // kernels, whose lanes are adjacent outputs)
    // lanes of one position are contiguous in memory: at least 16 x 16 bytes with four channels per lane,
    // at least 32 x 4 bytes with one (which is also what 32 ... 63 channels get when they are a multiple of 4)
    const bool v4 = vec && C >= 64;
    if (SW == 1 && DW == 1 && KW >= 2 && KW <= 9 && C >= 32) {
        // long runs once they still leave every SIMD a few wavefronts, short ones below that
        const int64_t CG = v4 ? C / 4 : C;
        const bool long_runs = N * OH * cdiv(OW, 8) * CG >= (int64_t)kDThreads * 256 * 4;
        const int RB = OH >= 4 ? 4 : 1;                          // output rows that share a workgroup (measured: 1, 4, 8)
        const int64_t items = N * cdiv(OH, RB) * RB * cdiv(OW, long_runs ? 8 : 4) * CG;
        const int64_t blocks = cdiv(items, kDThreads);
        if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
#define LG_DWR2(K_, T_, V_)                                                                                  \
        hipLaunchKernelGGL((dwconv_rows_kernel<K_, T_, V_>), dim3((unsigned)blocks), dim3(kDThreads), 0, s,   \
                           I, Kf, O, N, H, W, C, KH, SH, DH, OH, OW, accumulate, RB)
#define LG_DWR(K_)                                                                                            \
        if (KW == K_) {                                                                                      \
            if (v4 && long_runs)  LG_DWR2(K_, 8, 4);                                                         \
            else if (v4)          LG_DWR2(K_, 4, 4);                                                         \
            else if (long_runs)   LG_DWR2(K_, 8, 1);                                                         \
            else                  LG_DWR2(K_, 4, 1);                                                         \
            return launch_status();                                                                          \
        }
        LG_DWR(2) LG_DWR(3) LG_DWR(4) LG_DWR(5) LG_DWR(6) LG_DWR(7) LG_DWR(8) LG_DWR(9)
#undef LG_DWR
#undef LG_DWR2
    }
    // the same kernel at horizontal stride / dilation 2 for widths 3, 5, 7 (the 3 x 3 case with C % 4 == 0
    // went to the window kernels above): runs of 4 outputs
    if (SW <= 2 && DW <= 2 && (KW == 3 || KW == 5 || KW == 7) && C >= 32) {
        const int64_t CG = v4 ? C / 4 : C;
        const int RB = 1;                                        // measured: grouping rows costs 5-10 % at stride 2
        const int64_t items = N * cdiv(OH, RB) * RB * cdiv(OW, 4) * CG;
        const int64_t blocks = cdiv(items, kDThreads);
        if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
#define LG_DWS(K_, S_, D_)                                                                                    \
        if (KW == K_ && SW == S_ && DW == D_) {                                                              \
            if (v4)  hipLaunchKernelGGL((dwconv_rows_kernel<K_, 4, 4, S_, D_>), dim3((unsigned)blocks), dim3(kDThreads), 0, s, \
                                        I, Kf, O, N, H, W, C, KH, SH, DH, OH, OW, accumulate, RB);           \
            else     hipLaunchKernelGGL((dwconv_rows_kernel<K_, 4, 1, S_, D_>), dim3((unsigned)blocks), dim3(kDThreads), 0, s, \
                                        I, Kf, O, N, H, W, C, KH, SH, DH, OH, OW, accumulate, RB);           \
            return launch_status();                                                                          \
        }
        LG_DWS(3, 2, 1) LG_DWS(3, 1, 2) LG_DWS(3, 2, 2)
        LG_DWS(5, 2, 1) LG_DWS(5, 1, 2) LG_DWS(5, 2, 2)
        LG_DWS(7, 2, 1) LG_DWS(7, 1, 2) LG_DWS(7, 2, 2)
#undef LG_DWS
    }
    if (vec) {
        const int64_t blocks4 = cdiv(out_elems / 4, kDThreads);
        if (blocks4 > kMaxGrid) return LG_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(dwconv_general_vec4_kernel, dim3((unsigned)blocks4), dim3(kDThreads), 0, s,
                           I, Kf, O, N, H, W, C, KH, KW, SH, SW, DH, DW, OH, OW, accumulate);
        return launch_status();
    }
    const int64_t blocks = cdiv(out_elems, kDThreads);
    if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(dwconv_general_kernel, dim3((unsigned)blocks), dim3(kDThreads), 0, s,
                       I, Kf, O, N, H, W, C, KH, KW, SH, SW, DH, DW, OH, OW, accumulate);
    return launch_status();
}

}  // namespace lg

extern "C" int lg_dwconv1d_nwc_wc(const float* I, const float* Kf, float* O,
                                  int64_t N, int64_t W, int64_t C, int64_t KW,
                                  int64_t SW, int64_t DW, int accumulate, void* stream) {
    return lg::dwconv_dispatch(I, Kf, O, N, 1, W, C, 1, KW, 1, SW, 1, DW, accumulate, stream);
}

extern "C" int lg_dwconv2d_nhwc_hwc(const float* I, const float* Kf, float* O,
                                    int64_t N, int64_t H, int64_t W, int64_t C,
                                    int64_t KH, int64_t KW,
                                    int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                                    int accumulate, void* stream) {
    return lg::dwconv_dispatch(I, Kf, O, N, H, W, C, KH, KW, SH, SW, DH, DW, accumulate, stream);
}
