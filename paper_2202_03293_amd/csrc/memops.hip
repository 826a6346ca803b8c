// Copy2D and Transpose2D (Section 4.4): pure data movement, bound by HBM bandwidth.
#include "lg_common.hpp"

namespace lg {

constexpr int kCopyThreads = 256;
constexpr int kCopyUnroll = 4;   // 128-bit accesses in flight per lane

// out[i,j] = in[i,j].  VEC: rows are whole uint4s and everything is 16-byte aligned.
template <bool VEC>
__global__ __launch_bounds__(kCopyThreads) void copy2d_kernel(
    const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
    int64_t R, int64_t Cn, int64_t ld_in, int64_t ld_out) {
    constexpr int W = VEC ? 4 : 1;
    const int64_t per_row = Cn / W;
    const int64_t total = R * per_row;
    const int64_t base = (int64_t)blockIdx.x * (kCopyThreads * kCopyUnroll) + threadIdx.x;
    if constexpr (VEC) {
        uint4 v[kCopyUnroll];
        int64_t dst[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const int64_t idx = base + (int64_t)u * kCopyThreads;
            dst[u] = -1;
            if (idx < total) {
                const int64_t r = idx / per_row, c = idx - r * per_row;
                v[u] = *reinterpret_cast<const uint4*>(in + r * ld_in + 4 * c);
                dst[u] = r * ld_out + 4 * c;
            }
        }
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (dst[u] >= 0) *reinterpret_cast<uint4*>(out + dst[u]) = v[u];
    } else {
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const int64_t idx = base + (int64_t)u * kCopyThreads;
            if (idx < total) {
                const int64_t r = idx / per_row, c = idx - r * per_row;
                out[r * ld_out + c] = in[r * ld_in + c];
            }
        }
    }
}

constexpr int kTT = 64;          // transpose tile edge
constexpr int kTThreads = 256;

// out[j,i] = in[i,j] through a 64x64 LDS tile.  Row stride 65 words keeps both the row-wise
// writes and the column-wise reads of a wavefront on 32 distinct banks twice (the minimum for
// 64 lanes).  Global accesses are 128-bit on both sides when VEC.
template <bool VEC>
__global__ __launch_bounds__(kTThreads) void transpose_kernel(
    const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
    int64_t R, int64_t Cn, int64_t ld_in, int64_t ld_out, unsigned tiles_j, unsigned ntiles) {
    __shared__ uint32_t tile[kTT][kTT + 1];
    const unsigned id = xcd_contiguous_id(blockIdx.x, ntiles);
    const int64_t i0 = (int64_t)(id / tiles_j) * kTT;   // first input row of the tile
    const int64_t j0 = (int64_t)(id % tiles_j) * kTT;   // first input column
    const int t = threadIdx.x;
    if constexpr (VEC) {
        const int c4 = t % 16, rr = t / 16;
        uint4 v[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int r = it * 16 + rr;
            v[it] = make_uint4(0, 0, 0, 0);
            if (i0 + r < R && j0 + 4 * c4 < Cn)
                v[it] = *reinterpret_cast<const uint4*>(in + (i0 + r) * ld_in + j0 + 4 * c4);
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int r = it * 16 + rr;
            tile[r][4 * c4 + 0] = v[it].x;
            tile[r][4 * c4 + 1] = v[it].y;
            tile[r][4 * c4 + 2] = v[it].z;
            tile[r][4 * c4 + 3] = v[it].w;
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int orow = it * 16 + rr;     // column of the input tile = row of the output tile
            if (j0 + orow < Cn && i0 + 4 * c4 < R) {
                uint4 w;
                w.x = tile[4 * c4 + 0][orow];
                w.y = tile[4 * c4 + 1][orow];
                w.z = tile[4 * c4 + 2][orow];
                w.w = tile[4 * c4 + 3][orow];
                *reinterpret_cast<uint4*>(out + (j0 + orow) * ld_out + i0 + 4 * c4) = w;
            }
        }
    } else {
        const int c = t % 64, rr = t / 64;
#pragma unroll 4
        for (int it = 0; it < 16; ++it) {
            const int r = it * 4 + rr;
            if (i0 + r < R && j0 + c < Cn) tile[r][c] = in[(i0 + r) * ld_in + j0 + c];
        }
        __syncthreads();
#pragma unroll 4
        for (int it = 0; it < 16; ++it) {
            const int orow = it * 4 + rr;
            if (j0 + orow < Cn && i0 + c < R) out[(j0 + orow) * ld_out + i0 + c] = tile[c][orow];
        }
    }
}

}  // namespace lg

extern "C" int lg_copy2d(const float* in, float* out, int64_t R, int64_t Cn,
                         int64_t ld_in, int64_t ld_out, void* stream) {
    using namespace lg;
    if (R < 0 || Cn < 0 || ld_in < Cn || ld_out < Cn) return LG_ERR_INVALID_ARG;
    if (R == 0 || Cn == 0) return LG_OK;
    if (!in || !out) return LG_ERR_INVALID_ARG;
    if (overlaps(in, ((R - 1) * ld_in + Cn) * 4, out, ((R - 1) * ld_out + Cn) * 4)) return LG_ERR_INVALID_ARG;
    if (ld_in == Cn && ld_out == Cn) {   // dense: one long row
        Cn *= R; R = 1; ld_in = ld_out = Cn;
    }
    const bool vec = (Cn % 4 == 0) && (ld_in % 4 == 0) && (ld_out % 4 == 0) && aligned16(in) && aligned16(out);
    const int64_t items = vec ? R * (Cn / 4) : R * Cn;
    const int64_t blocks = cdiv(items, kCopyThreads * kCopyUnroll);
    if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto* i32 = reinterpret_cast<const uint32_t*>(in);
    auto* o32 = reinterpret_cast<uint32_t*>(out);
    if (vec) hipLaunchKernelGGL(copy2d_kernel<true>, dim3((unsigned)blocks), dim3(kCopyThreads), 0, s, i32, o32, R, Cn, ld_in, ld_out);
    else     hipLaunchKernelGGL(copy2d_kernel<false>, dim3((unsigned)blocks), dim3(kCopyThreads), 0, s, i32, o32, R, Cn, ld_in, ld_out);
    return launch_status();
}

extern "C" int lg_transpose(const float* in, float* out, int64_t R, int64_t Cn,
                            int64_t ld_in, int64_t ld_out, void* stream) {
    using namespace lg;
    if (R < 0 || Cn < 0 || ld_in < Cn || ld_out < R) return LG_ERR_INVALID_ARG;
    if (R == 0 || Cn == 0) return LG_OK;
    if (!in || !out) return LG_ERR_INVALID_ARG;
    if (overlaps(in, ((R - 1) * ld_in + Cn) * 4, out, ((Cn - 1) * ld_out + R) * 4)) return LG_ERR_INVALID_ARG;
    const int64_t ti = cdiv(R, kTT), tj = cdiv(Cn, kTT);
    if (ti * tj > kMaxGrid || tj > kMaxGrid) return LG_ERR_UNSUPPORTED;
    const bool vec = (Cn % 4 == 0) && (R % 4 == 0) && (ld_in % 4 == 0) && (ld_out % 4 == 0) &&
                     aligned16(in) && aligned16(out);
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto* i32 = reinterpret_cast<const uint32_t*>(in);
    auto* o32 = reinterpret_cast<uint32_t*>(out);
    const unsigned nt = (unsigned)(ti * tj);
    if (vec) hipLaunchKernelGGL(transpose_kernel<true>, dim3(nt), dim3(kTThreads), 0, s, i32, o32, R, Cn, ld_in, ld_out, (unsigned)tj, nt);
    else     hipLaunchKernelGGL(transpose_kernel<false>, dim3(nt), dim3(kTThreads), 0, s, i32, o32, R, Cn, ld_in, ld_out, (unsigned)tj, nt);
    return launch_status();
}
