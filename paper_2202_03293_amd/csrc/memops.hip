// Copy2D and Transpose2D (Section 4.4): pure data movement, bound by HBM bandwidth.
#include "lg_common.hpp"

namespace lg {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kCopyThreads = 256;
// 128-bit accesses per lane.  One: many small workgroups that each move 4 KiB and retire keep the
// stream strictly sequential across the chip (measured on 8192 x 8192, cold, back to back:
// 1 / 2 / 4 words per lane 82.7 / 86.8 / 86.8 us with the non-temporal hints on both sides).
constexpr int kCopyUnroll = 1;
constexpr int kTrLanesPerRow = 32;   // lanes side by side on a tile row of the transpose: 512 contiguous bytes per half wavefront

// out[i,j] = in[i,j].  VEC: rows are whole 128-bit words and everything is 16-byte aligned; the
// stream is marked non-temporal on both sides (nothing is reused, keep it out of the caches).
// FLAT: both sides are dense (row pitch = row length), so the matrix is one long row and no lane
// has to divide its index by the row length (a 64-bit division costs more than the copy of a small
// matrix).
template <bool VEC, bool STREAM = true, bool FLAT = false>
__global__ __launch_bounds__(kCopyThreads) void copy2d_kernel(
    const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
    int64_t R, int64_t Cn, int64_t ld_in, int64_t ld_out) {
    constexpr int W = VEC ? 4 : 1;
    const int64_t per_row = Cn / W;
    const int64_t total = R * per_row;
    const int64_t base = (int64_t)blockIdx.x * (kCopyThreads * kCopyUnroll) + threadIdx.x;
    if constexpr (VEC) {
        u32x4 v[kCopyUnroll];
        int64_t dst[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const int64_t idx = base + (int64_t)u * kCopyThreads;
            dst[u] = -1;
            if (idx < total) {
                const int64_t r = FLAT ? 0 : idx / per_row, c = idx - r * per_row;
                const u32x4* src = reinterpret_cast<const u32x4*>(in + r * ld_in + 4 * c);
                if constexpr (STREAM) v[u] = __builtin_nontemporal_load(src); else v[u] = *src;
                dst[u] = r * ld_out + 4 * c;
            }
        }
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (dst[u] >= 0) {
                if constexpr (STREAM) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4*>(out + dst[u]));
                else *reinterpret_cast<u32x4*>(out + dst[u]) = v[u];
            }
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

// out[j,i] = in[i,j] through a TS x TS LDS tile (TS = 64 or 128) by THREADS lanes.
//
// Global side: 32 lanes (16 for TS = 64) cover the TS*4 contiguous bytes of a tile row, on both
// sides, so a wavefront's access is two 512-byte pieces rather than four of 256 (measured on
// 8192 x 8192, cold, back to back: 101.8 -> 95.2 us).  LDS side: row stride TS+1 words, and the
// order in which a lane walks its four words rotated by lane group (see `rot` below), keep the
// row-wise writes and the column-wise reads of a wavefront on 32 distinct banks twice, the minimum
// for 64 lanes.  Tiles are visited along diagonals so that workgroups running together
// differ in both row and column block: their strided accesses then do not pile onto the same
// memory channels.  The walk follows the input rows for square and tall inputs and the output rows
// for wide ones (measured, 128x128 tiles: 1024 x 65536 129 -> 106 us, 4096 x 16384 122 -> 115 us;
// tall and square inputs lose 2-10 % with the other walk).  The XCD-contiguous id order is deliberately NOT used here (measured slower:
// nothing is shared between tiles, and spreading neighbours over all L2s is what helps).
// element offsets of batch (b0, b1): b0 * in0 + b1 * in1 into the input, likewise the output
struct BatchStrides { int64_t in0, in1, out0, out1; };

template <int TS, int THREADS, bool VEC>
__global__ __launch_bounds__(THREADS) void transpose_kernel(
    const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
    int64_t R, int64_t Cn, int64_t ld_in, int64_t ld_out, unsigned tiles_i, unsigned tiles_j, int walk_columns,
    BatchStrides bs) {
    extern __shared__ uint32_t tile[];              // [TS][TS + 1]
    constexpr int S = TS + 1;
    in += blockIdx.z * bs.in0 + blockIdx.y * bs.in1;      // batch (b0, b1) = (blockIdx.z, blockIdx.y)
    out += blockIdx.z * bs.out0 + blockIdx.y * bs.out1;
    unsigned ti, tj;
    if (walk_columns) {          // consecutive workgroups share output rows (wide inputs)
        tj = blockIdx.x / tiles_i;
        ti = (blockIdx.x % tiles_i + tj) % tiles_i;
    } else {                     // consecutive workgroups share input rows
        ti = blockIdx.x / tiles_j;
        tj = (blockIdx.x % tiles_j + ti) % tiles_j;
    }
    const int64_t i0 = (int64_t)ti * TS;            // first input row of the tile
    const int64_t j0 = (int64_t)tj * TS;            // first input column
    const int t = threadIdx.x;
    if constexpr (VEC) {
        constexpr int LPR = (kTrLanesPerRow * 4 <= TS) ? kTrLanesPerRow : TS / 4;   // lanes side by side on a row
        constexpr int CW = 4 * LPR;                 // columns they cover
        constexpr int RP = THREADS / LPR;           // rows per pass
        constexpr int NL = (TS / RP) * (TS / CW);   // 128-bit words per lane
        const int c4 = t % LPR, rr = t / LPR;
        // LDS position of tile element (r, c): rows and columns are de-interleaved by four -- row r sits
        // at slot (r % 4) * TS/4 + r / 4, column c likewise -- so that the lanes of a row, whose words in
        // step e are the columns 4*c4 + e, and the lanes of a column, whose words are the rows 4*c4 + e,
        // both land in consecutive slots, i.e. on distinct banks (the row stride S is odd).
        constexpr int Q = TS / 4;
        u32x4 v[NL];
        int k = 0;
#pragma unroll
        for (int rp = 0; rp < TS / RP; ++rp)
#pragma unroll
            for (int cc = 0; cc < TS / CW; ++cc) {
                const int64_t gi = i0 + rp * RP + rr, gj = j0 + cc * CW + 4 * c4;
                v[k] = u32x4{0, 0, 0, 0};
                if (gi < R && gj < Cn) {
                    const u32x4* src = reinterpret_cast<const u32x4*>(in + gi * ld_in + gj);
                    v[k] = *src;
                }
                ++k;
            }
        k = 0;
#pragma unroll
        for (int rp = 0; rp < TS / RP; ++rp)
#pragma unroll
            for (int cc = 0; cc < TS / CW; ++cc) {
                const int r = rp * RP + rr;
                uint32_t* p = tile + ((r & 3) * Q + (r >> 2)) * S + cc * (CW / 4) + c4;
                p[0] = v[k].x; p[Q] = v[k].y; p[2 * Q] = v[k].z; p[3 * Q] = v[k].w;
                ++k;
            }
        __syncthreads();
#pragma unroll
        for (int rp = 0; rp < TS / RP; ++rp)
#pragma unroll
            for (int cc = 0; cc < TS / CW; ++cc) {
                const int orow = rp * RP + rr;      // column of the input tile = row of the output tile
                const int ic = cc * CW + 4 * c4;    // row of the input tile = column of the output tile
                if (j0 + orow < Cn && i0 + ic < R) {
                    const uint32_t* q = tile + (cc * (CW / 4) + c4) * S + (orow & 3) * Q + (orow >> 2);
                    u32x4 w;
                    w.x = q[0];
                    w.y = q[Q * S];
                    w.z = q[2 * Q * S];
                    w.w = q[3 * Q * S];
                    u32x4* dst = reinterpret_cast<u32x4*>(out + (j0 + orow) * ld_out + i0 + ic);
                    *dst = w;
                }
            }
    } else {
        constexpr int RP = THREADS / TS;
        const int c = t % TS, rr = t / TS;
        constexpr int NP = TS / RP;                 // elements per lane, all requested before the first lands in LDS
        uint32_t v[NP];
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const int r = rr + k * RP;
            v[k] = 0;
            if (i0 + r < R && j0 + c < Cn) v[k] = in[(i0 + r) * ld_in + j0 + c];
        }
#pragma unroll
        for (int k = 0; k < NP; ++k) tile[(rr + k * RP) * S + c] = v[k];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const int orow = rr + k * RP;
            if (j0 + orow < Cn && i0 + c < R) out[(j0 + orow) * ld_out + i0 + c] = tile[c * S + orow];
        }
    }
}

template <int TS, int THREADS, bool VEC>
static int launch_transpose(const uint32_t* in, uint32_t* out, int64_t R, int64_t Cn,
                            int64_t ld_in, int64_t ld_out, int64_t B0, int64_t B1, BatchStrides bs, hipStream_t s) {
    const int64_t ti = cdiv(R, TS), tj = cdiv(Cn, TS);
    if (ti * tj > kMaxGrid || B0 > 65535 || B1 > 65535) return LG_ERR_UNSUPPORTED;
    constexpr size_t lds = (size_t)TS * (TS + 1) * sizeof(uint32_t);
    static DeviceFlags configured = {};
    allow_dynamic_lds(reinterpret_cast<const void*>(&transpose_kernel<TS, THREADS, VEC>), lds, configured);
    hipLaunchKernelGGL((transpose_kernel<TS, THREADS, VEC>), dim3((unsigned)(ti * tj), (unsigned)B1, (unsigned)B0),
                       dim3(THREADS), lds, s, in, out, R, Cn, ld_in, ld_out, (unsigned)ti, (unsigned)tj,
                       Cn > R ? 1 : 0, bs);
    return launch_status();
}

}  // namespace lg

extern "C" int lg_copy2d(const float* in, float* out, int64_t R, int64_t Cn,
                         int64_t ld_in, int64_t ld_out, void* stream) {
    using namespace lg;
    if (R < 0 || Cn < 0 || ld_in < Cn || ld_out < Cn) return LG_ERR_INVALID_ARG;
    if (R == 0 || Cn == 0) return LG_OK;
    if (!in || !out) return LG_ERR_INVALID_ARG;
    if (overlaps(in, ((R - 1) * ld_in + Cn) * 4, out, ((R - 1) * ld_out + Cn) * 4)) return LG_ERR_INVALID_ARG;
    hipStream_t s = begin_call(stream);
    if (ld_in == Cn && ld_out == Cn) {   // dense: one long row
        Cn *= R; R = 1; ld_in = ld_out = Cn;
        // a long dense array whose length is not a multiple of 4: the 128-bit body, then the last 1-3 floats
        if (Cn % 4 != 0 && Cn >= (1 << 20) && aligned16(in) && aligned16(out)) {
            const int64_t body = Cn - Cn % 4;
            const int rc = lg_copy2d(in, out, 1, body, body, body, stream);
            if (rc != LG_OK) return rc;
            hipLaunchKernelGGL((lg::copy2d_kernel<false, false>), dim3(1), dim3(lg::kCopyThreads), 0, s,
                               reinterpret_cast<const uint32_t*>(in + body), reinterpret_cast<uint32_t*>(out + body),
                               (int64_t)1, Cn - body, Cn - body, Cn - body);
            return lg::launch_status();
        }
    }
    const bool vec = (Cn % 4 == 0) && (ld_in % 4 == 0) && (ld_out % 4 == 0) && aligned16(in) && aligned16(out);
    const int64_t items = vec ? R * (Cn / 4) : R * Cn;
    const int64_t blocks = cdiv(items, kCopyThreads * kCopyUnroll);
    if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
    auto* i32 = reinterpret_cast<const uint32_t*>(in);
    auto* o32 = reinterpret_cast<uint32_t*>(out);
    // Past what the last-level cache holds nothing of the stream is worth keeping; a small copy is
    // usually read again by the next kernel, and is faster itself through the caches.
    const bool stream_hint = 2 * R * Cn * 4 > ((int64_t)200 << 20);      // 256 MB of last-level cache on this part
    const bool flat = ld_in == Cn && ld_out == Cn;
    if (vec && stream_hint && flat) hipLaunchKernelGGL((copy2d_kernel<true, true, true>), dim3((unsigned)blocks), dim3(kCopyThreads), 0, s, i32, o32, R, Cn, ld_in, ld_out);
    else if (vec && stream_hint) hipLaunchKernelGGL((copy2d_kernel<true, true, false>), dim3((unsigned)blocks), dim3(kCopyThreads), 0, s, i32, o32, R, Cn, ld_in, ld_out);
    else if (vec && flat) hipLaunchKernelGGL((copy2d_kernel<true, false, true>), dim3((unsigned)blocks), dim3(kCopyThreads), 0, s, i32, o32, R, Cn, ld_in, ld_out);
    else if (vec) hipLaunchKernelGGL((copy2d_kernel<true, false, false>), dim3((unsigned)blocks), dim3(kCopyThreads), 0, s, i32, o32, R, Cn, ld_in, ld_out);
    else     hipLaunchKernelGGL((copy2d_kernel<false, false>), dim3((unsigned)blocks), dim3(kCopyThreads), 0, s, i32, o32, R, Cn, ld_in, ld_out);
    return launch_status();
}

namespace lg {

// Transpose of a matrix with very few rows or very few columns (a vector, three interleaved
// channels): an LDS tile would be almost empty.  One element per lane, walking the side whose rows
// are the short ones in memory order, so that the other side is a handful of contiguous streams.
// BY_OUT: lanes enumerate the output (R small: out rows are R long); else the input (Cn small).
template <bool BY_OUT>
__global__ __launch_bounds__(256) void transpose_thin_kernel(
    const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
    int64_t R, int64_t Cn, int64_t ld_in, int64_t ld_out, BatchStrides bs) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= R * Cn) return;
    in += (int64_t)blockIdx.z * bs.in0 + (int64_t)blockIdx.y * bs.in1;      // batch (b0, b1) = (z, y)
    out += (int64_t)blockIdx.z * bs.out0 + (int64_t)blockIdx.y * bs.out1;
    const int64_t minor = BY_OUT ? R : Cn;
    int64_t major, rem;
    if (R * Cn < ((int64_t)1 << 32)) {             // 32-bit division when it fits: several times cheaper
        const uint32_t q = (uint32_t)idx / (uint32_t)minor;
        major = q; rem = (uint32_t)idx - q * (uint32_t)minor;
    } else {
        major = idx / minor; rem = idx - major * minor;
    }
    const int64_t i = BY_OUT ? rem : major, j = BY_OUT ? major : rem;
    out[j * ld_out + i] = in[i * ld_in + j];
}

static int transpose_dispatch(const float* in, float* out, int64_t R, int64_t Cn, int64_t ld_in, int64_t ld_out,
                              int64_t B0, int64_t B1, BatchStrides bs, bool vec, void* stream) {
    hipStream_t s = begin_call(stream);
    auto* i32 = reinterpret_cast<const uint32_t*>(in);
    auto* o32 = reinterpret_cast<uint32_t*>(out);
    if (R < 16 || Cn < 16) {                       // e.g. NHWC <-> NCHW with three channels, as a batch over N
        const int64_t blocks = cdiv(R * Cn, 256);
        if (blocks > kMaxGrid || B0 > 65535 || B1 > 65535) return LG_ERR_UNSUPPORTED;
        const dim3 grid((unsigned)blocks, (unsigned)B1, (unsigned)B0);
        if (R <= Cn) hipLaunchKernelGGL(transpose_thin_kernel<true>, grid, dim3(256), 0, s, i32, o32, R, Cn, ld_in, ld_out, bs);
        else         hipLaunchKernelGGL(transpose_thin_kernel<false>, grid, dim3(256), 0, s, i32, o32, R, Cn, ld_in, ld_out, bs);
        return launch_status();
    }
    // 128x128 tiles once they still give every CU several workgroups, 64x64 below that
    const bool big = cdiv(R, 128) * cdiv(Cn, 128) * B0 * B1 >= 1024 && R >= 128 && Cn >= 128;
    if (vec && big) return launch_transpose<128, 1024, true>(i32, o32, R, Cn, ld_in, ld_out, B0, B1, bs, s);
    if (vec)        return launch_transpose<64, 256, true>(i32, o32, R, Cn, ld_in, ld_out, B0, B1, bs, s);
    return launch_transpose<64, 256, false>(i32, o32, R, Cn, ld_in, ld_out, B0, B1, bs, s);
}

}  // namespace lg

extern "C" int lg_transpose(const float* in, float* out, int64_t R, int64_t Cn,
                            int64_t ld_in, int64_t ld_out, void* stream) {
    using namespace lg;
    if (R < 0 || Cn < 0 || ld_in < Cn || ld_out < R) return LG_ERR_INVALID_ARG;
    if (R == 0 || Cn == 0) return LG_OK;
    if (!in || !out) return LG_ERR_INVALID_ARG;
    if (overlaps(in, ((R - 1) * ld_in + Cn) * 4, out, ((Cn - 1) * ld_out + R) * 4)) return LG_ERR_INVALID_ARG;
    const bool vec = (Cn % 4 == 0) && (R % 4 == 0) && (ld_in % 4 == 0) && (ld_out % 4 == 0) &&
                     aligned16(in) && aligned16(out);
    return transpose_dispatch(in, out, R, Cn, ld_in, ld_out, 1, 1, BatchStrides{0, 0, 0, 0}, vec, stream);
}

extern "C" int lg_transpose_batched(const float* in, float* out, int64_t R, int64_t Cn,
                                    int64_t ld_in, int64_t ld_out,
                                    int64_t B0, int64_t B1,
                                    int64_t in_stride0, int64_t in_stride1,
                                    int64_t out_stride0, int64_t out_stride1, void* stream) {
    using namespace lg;
    if (R < 0 || Cn < 0 || B0 < 0 || B1 < 0 || ld_in < Cn || ld_out < R) return LG_ERR_INVALID_ARG;
    if (in_stride0 < 0 || in_stride1 < 0 || out_stride0 < 0 || out_stride1 < 0) return LG_ERR_INVALID_ARG;
    if (R == 0 || Cn == 0 || B0 == 0 || B1 == 0) return LG_OK;
    if (!in || !out) return LG_ERR_INVALID_ARG;
    const int64_t in_span = (B0 - 1) * in_stride0 + (B1 - 1) * in_stride1 + (R - 1) * ld_in + Cn;
    const int64_t out_span = (B0 - 1) * out_stride0 + (B1 - 1) * out_stride1 + (Cn - 1) * ld_out + R;
    if (overlaps(in, in_span * 4, out, out_span * 4)) return LG_ERR_INVALID_ARG;
    const bool vec = (Cn % 4 == 0) && (R % 4 == 0) && (ld_in % 4 == 0) && (ld_out % 4 == 0) &&
                     (in_stride0 % 4 == 0) && (in_stride1 % 4 == 0) && (out_stride0 % 4 == 0) &&
                     (out_stride1 % 4 == 0) && aligned16(in) && aligned16(out);
    return transpose_dispatch(in, out, R, Cn, ld_in, ld_out, B0, B1,
                              BatchStrides{in_stride0, in_stride1, out_stride0, out_stride1}, vec, stream);
}
