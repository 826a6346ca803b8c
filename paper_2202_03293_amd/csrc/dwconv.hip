// Depthwise convolutions (Section 4.7): no contraction across channels, so no matrix cores;
// K_w (or K_h*K_w) FMAs per output element against 8 bytes of traffic -> HBM-bound.
//
// Fast kernels: a lane owns 4 adjacent channels (one 128-bit access) and a run of output
// positions, keeps the input window in registers so each input element is loaded once per
// lane, and neighbouring lanes/workgroups share the halo through L2.  General kernels cover
// any stride, dilation, filter size and channel count one output element per lane.
#include "lg_common.hpp"

namespace lg {

constexpr int kDThreads = 256;

typedef float f32x4 __attribute__((ext_vector_type(4)));

// 128-bit streaming store: the output is written once and not read again by this kernel.
__device__ __forceinline__ void store_stream4(float* p, const float4 v) {
    __builtin_nontemporal_store(f32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4*>(p));
}

__device__ __forceinline__ float4 fma4(const float4 a, const float4 b, const float4 c) {
    return make_float4(fmaf(a.x, b.x, c.x), fmaf(a.y, b.y, c.y), fmaf(a.z, b.z, c.z), fmaf(a.w, b.w, c.w));
}

// 1-D, stride 1, dilation 1, C % 4 == 0.  Lane -> (n, run of TW outputs, 4 channels); channels vary
// fastest across lanes so a wavefront reads 1 KiB contiguous per input position.
template <int KW, int TW>
__global__ __launch_bounds__(kDThreads) void dwconv1d_s1_kernel(
    const float* __restrict__ I, const float* __restrict__ Kf, float* __restrict__ O,
    int64_t N, int64_t W, int64_t C, int64_t OW, int accumulate, unsigned nblocks) {
    const int64_t C4 = C / 4;
    const int64_t runs = (OW + TW - 1) / TW;
    const int64_t total = N * runs * C4;
    const int64_t idx = (int64_t)xcd_contiguous_id(blockIdx.x, nblocks) * kDThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t c4 = idx % C4;
    const int64_t run = (idx / C4) % runs;
    const int64_t n = idx / (C4 * runs);
    const int64_t w0 = run * TW;
    const int nout = (OW - w0 < TW) ? (int)(OW - w0) : TW;
    float4 k[KW];
#pragma unroll
    for (int i = 0; i < KW; ++i) k[i] = *reinterpret_cast<const float4*>(Kf + i * C + 4 * c4);
    const float* ip = I + (n * W + w0) * C + 4 * c4;
    float* op = O + (n * OW + w0) * C + 4 * c4;
    float4 x[TW + KW - 1];
#pragma unroll
    for (int i = 0; i < TW + KW - 1; ++i) {
        x[i] = make_float4(0, 0, 0, 0);
        if (i < nout + KW - 1) x[i] = *reinterpret_cast<const float4*>(ip + (int64_t)i * C);
    }
#pragma unroll
    for (int o = 0; o < TW; ++o) {
        if (o < nout) {
            float4 acc = accumulate ? *reinterpret_cast<const float4*>(op + (int64_t)o * C) : make_float4(0, 0, 0, 0);
            // the initial accumulator enters last so that overwrite and accumulate share the k-sum
            float4 s = make_float4(0, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < KW; ++i) s = fma4(x[o + i], k[i], s);
            if (accumulate) { s.x += acc.x; s.y += acc.y; s.z += acc.z; s.w += acc.w; }
            *reinterpret_cast<float4*>(op + (int64_t)o * C) = s;
        }
    }
}

// 2-D, stride 1, dilation 1, C % 4 == 0.  Lane -> (n, TH x TW output patch, 4 channels).  The whole
// (TH+KH-1) x (TW+KW-1) input patch is requested before any arithmetic, so a lane exposes one
// memory latency, not one per row (measured 27 -> 19 us on the 8x114x114x96 workload against a
// rolling row window).  Outputs are streamed with non-temporal stores.  Plain workgroup order:
// the XCD-contiguous order measured slightly slower here.
template <int KH, int KW, int TH, int TW>
__global__ __launch_bounds__(kDThreads) void dwconv2d_s1_kernel(
    const float* __restrict__ I, const float* __restrict__ Kf, float* __restrict__ O,
    int64_t N, int64_t H, int64_t W, int64_t C, int64_t OH, int64_t OW, int accumulate) {
    const int64_t C4 = C / 4;
    const int64_t pw = (OW + TW - 1) / TW, ph = (OH + TH - 1) / TH;
    const int64_t total = N * ph * pw * C4;
    const int64_t idx = (int64_t)blockIdx.x * kDThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t c4 = idx % C4;
    const int64_t bw = (idx / C4) % pw;
    const int64_t bh = (idx / (C4 * pw)) % ph;
    const int64_t n = idx / (C4 * pw * ph);
    const int64_t h0 = bh * TH, w0 = bw * TW;
    const int nh = (OH - h0 < TH) ? (int)(OH - h0) : TH;
    const int nw = (OW - w0 < TW) ? (int)(OW - w0) : TW;
    const float* ip = I + ((n * H + h0) * W + w0) * C + 4 * c4;
    float* op = O + ((n * OH + h0) * OW + w0) * C + 4 * c4;
    float4 x[TH + KH - 1][TW + KW - 1];
#pragma unroll
    for (int r = 0; r < TH + KH - 1; ++r)
#pragma unroll
        for (int i = 0; i < TW + KW - 1; ++i) {
            x[r][i] = make_float4(0, 0, 0, 0);
            if (r < nh + KH - 1 && i < nw + KW - 1)
                x[r][i] = *reinterpret_cast<const float4*>(ip + ((int64_t)r * W + i) * C);
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
                    for (int b = 0; b < KW; ++b) s = fma4(x[r + a][o + b], k[a][b], s);
                float* q = op + ((int64_t)r * OW + o) * C;
                if (accumulate) {
                    const float4 acc = *reinterpret_cast<const float4*>(q);
                    s.x += acc.x; s.y += acc.y; s.z += acc.z; s.w += acc.w;
                }
                store_stream4(q, s);
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
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool unit = SH == 1 && SW == 1 && DH == 1 && DW == 1;
    const bool vec = (C % 4 == 0) && aligned16(I) && aligned16(Kf) && aligned16(O);
    if (unit && vec && KH == 1 && KW == 3) {
        constexpr int TW = 4;    // measured best: short runs, many lanes in flight
        // H rows of a 1-D problem are independent images: fold them into N
        const int64_t NN = N * H;
        const int64_t items = NN * cdiv(OW, TW) * (C / 4);
        const int64_t blocks = cdiv(items, kDThreads);
        if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((dwconv1d_s1_kernel<3, TW>), dim3((unsigned)blocks), dim3(kDThreads), 0, s,
                           I, Kf, O, NN, W, C, OW, accumulate, (unsigned)blocks);
        return launch_status();
    }
    if (unit && vec && KH == 3 && KW == 3) {
        constexpr int TH = 4, TW = 2;   // small patches: the problem must fill 256 CUs
        const int64_t items = N * cdiv(OH, TH) * cdiv(OW, TW) * (C / 4);
        const int64_t blocks = cdiv(items, kDThreads);
        if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((dwconv2d_s1_kernel<3, 3, TH, TW>), dim3((unsigned)blocks), dim3(kDThreads), 0, s,
                           I, Kf, O, N, H, W, C, OH, OW, accumulate);
        return launch_status();
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
