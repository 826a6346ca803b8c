// Matrix-pipe yardstick: what the fp32 MFMA units sustain when nothing else is in the way.  The
// counterpart of lg_copy2d for the compute-bound kernels: the paper quotes its bandwidth-bound
// kernels against a measured copy and its compute-bound ones against the machine's theoretical
// peak (Section 4.3); this gives the measured figure beside the theoretical one.
#include "lg_common.hpp"

namespace lg {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 256;                 // one wavefront per SIMD of a CU
constexpr int kProbeGroups = 2 * 256;              // two workgroups per CU: two wavefronts per SIMD
constexpr int kProbeChains = 4;                    // independent accumulators per wavefront
constexpr int64_t kProbeMaxIters = 1 << 22;

// Every wavefront issues iters * kProbeChains 32x32x2 MFMAs on registers only; the chains are
// independent, so the pipe never waits for a result.  Operands are small lane-dependent values
// (bits that toggle like real data, sums that stay far from overflow).
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(float* __restrict__ out, int iters) {
    const unsigned lane = threadIdx.x % kWave;
    const float a = (float)((int)((lane * 37u + blockIdx.x * 11u) % 127u) - 63) * (1.0f / 65536.0f);
    const float b = (float)((int)((lane * 53u + threadIdx.x / kWave * 29u) % 113u) - 56) * (1.0f / 65536.0f);
    floatx16 acc[kProbeChains];
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kProbeChains; ++c)
            acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[c][i];
    out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

}  // namespace lg

extern "C" int64_t lg_mfma_probe_out_elems(void) { return (int64_t)lg::kProbeGroups * lg::kProbeThreads; }

extern "C" double lg_mfma_probe_flops(int64_t iters) {
    if (iters < 0) return 0.0;
    // 32 * 32 * 2 multiply-adds per MFMA
    return (double)lg::kProbeGroups * (lg::kProbeThreads / lg::kWave) * (double)iters * lg::kProbeChains * (32.0 * 32.0 * 2.0 * 2.0);
}

extern "C" int lg_mfma_probe(float* out, int64_t out_elems, int64_t iters, void* stream) {
    using namespace lg;
    if (iters < 0 || iters > kProbeMaxIters || out_elems < 0) return LG_ERR_INVALID_ARG;
    if (!out || out_elems < lg_mfma_probe_out_elems()) return LG_ERR_INVALID_ARG;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(kProbeGroups), dim3(kProbeThreads), 0,
                       begin_call(stream), out, (int)iters);
    return launch_status();
}
