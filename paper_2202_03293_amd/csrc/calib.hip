// Calibration kernels: the matrix-pipe yardstick and the HBM stream yardsticks.
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

// ---- HBM stream yardsticks ---------------------------------------------------------------------
// What the memory system sustains for the three access mixes the memory-bound ops are made of: a
// pure read stream (the reductions), a pure write stream, and a copy (transpose, depthwise
// convolution).  Every lane moves U float4, THREADS apart, of its workgroup's contiguous chunk; the
// launch shape and the cache hints are parameters so that the sweep behind the quoted ceilings can be
// repeated.  The read kernel adds what it loads and stores only if the sum is NaN, which finite
// inputs never produce: the loads stay, the stores cost nothing.
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int U, bool NT>
__global__ __launch_bounds__(1024) void stream_read_kernel(const f32x4* __restrict__ in, float* __restrict__ out, int64_t n4) {
    const int64_t base = (int64_t)blockIdx.x * (blockDim.x * U) + threadIdx.x;
    f32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t i = base + (int64_t)u * blockDim.x;
        v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (i < n4) v[u] = NT ? __builtin_nontemporal_load(in + i) : in[i];
    }
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) s += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    if (s != s) out[threadIdx.x] = s;
}

template <int U, bool NT>
__global__ __launch_bounds__(1024) void stream_write_kernel(f32x4* __restrict__ out, int64_t n4) {
    const int64_t base = (int64_t)blockIdx.x * (blockDim.x * U) + threadIdx.x;
    const f32x4 v = f32x4{1.f, 2.f, 3.f, 4.f};
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t i = base + (int64_t)u * blockDim.x;
        if (i < n4) {
            if (NT) __builtin_nontemporal_store(v, out + i); else out[i] = v;
        }
    }
}

template <int U, bool NTL, bool NTS>
__global__ __launch_bounds__(1024) void stream_copy_kernel(const f32x4* __restrict__ in, f32x4* __restrict__ out, int64_t n4) {
    const int64_t base = (int64_t)blockIdx.x * (blockDim.x * U) + threadIdx.x;
    f32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t i = base + (int64_t)u * blockDim.x;
        if (i < n4) v[u] = NTL ? __builtin_nontemporal_load(in + i) : in[i];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t i = base + (int64_t)u * blockDim.x;
        if (i < n4) {
            if (NTS) __builtin_nontemporal_store(v[u], out + i); else out[i] = v[u];
        }
    }
}

template <int U>
static void launch_stream(int mode, const f32x4* in, f32x4* out, int64_t n4, int threads, int hint, unsigned blocks, hipStream_t s) {
    const dim3 g(blocks), b(threads);
    const bool ntl = hint & 1, nts = hint & 2;
    if (mode == 0) {
        if (ntl) hipLaunchKernelGGL((stream_read_kernel<U, true>), g, b, 0, s, in, reinterpret_cast<float*>(out), n4);
        else     hipLaunchKernelGGL((stream_read_kernel<U, false>), g, b, 0, s, in, reinterpret_cast<float*>(out), n4);
    } else if (mode == 1) {
        if (nts) hipLaunchKernelGGL((stream_write_kernel<U, true>), g, b, 0, s, out, n4);
        else     hipLaunchKernelGGL((stream_write_kernel<U, false>), g, b, 0, s, out, n4);
    } else {
        if (ntl && nts)  hipLaunchKernelGGL((stream_copy_kernel<U, true, true>), g, b, 0, s, in, out, n4);
        else if (ntl)    hipLaunchKernelGGL((stream_copy_kernel<U, true, false>), g, b, 0, s, in, out, n4);
        else if (nts)    hipLaunchKernelGGL((stream_copy_kernel<U, false, true>), g, b, 0, s, in, out, n4);
        else             hipLaunchKernelGGL((stream_copy_kernel<U, false, false>), g, b, 0, s, in, out, n4);
    }
}

}  // namespace lg

extern "C" int lg_stream_probe(int mode, const float* in, float* out, int64_t n, int threads, int unroll, int hint,
                               void* stream) {
    using namespace lg;
    if (mode < 0 || mode > 2 || n < 0 || n % 4 != 0 || hint < 0 || hint > 3) return LG_ERR_INVALID_ARG;
    if (threads != 256 && threads != 512 && threads != 1024) return LG_ERR_INVALID_ARG;
    if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8) return LG_ERR_INVALID_ARG;
    if (n == 0) return LG_OK;
    if (!out || (mode != 1 && !in) || !aligned16(out) || (mode != 1 && !aligned16(in))) return LG_ERR_INVALID_ARG;
    // the read probe's `out` is a sink of at least 1024 floats; the others write n floats
    if (mode != 1 && overlaps(in, n * 4, out, (mode == 0 ? 1024 : n) * 4)) return LG_ERR_INVALID_ARG;
    const int64_t n4 = n / 4, blocks = cdiv(n4, (int64_t)threads * unroll);
    if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
    hipStream_t s = begin_call(stream);
    const f32x4* i4 = reinterpret_cast<const f32x4*>(in);
    f32x4* o4 = reinterpret_cast<f32x4*>(out);
    switch (unroll) {
        case 1: launch_stream<1>(mode, i4, o4, n4, threads, hint, (unsigned)blocks, s); break;
        case 2: launch_stream<2>(mode, i4, o4, n4, threads, hint, (unsigned)blocks, s); break;
        case 4: launch_stream<4>(mode, i4, o4, n4, threads, hint, (unsigned)blocks, s); break;
        default: launch_stream<8>(mode, i4, o4, n4, threads, hint, (unsigned)blocks, s); break;
    }
    return launch_status();
}

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
