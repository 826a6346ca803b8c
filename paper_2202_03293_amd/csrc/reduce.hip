// RowRed2D and ColRed2D (Section 4.4): HBM-bound read streams.
//
// Both keep every fp32 running sum short: a lane adds at most a few dozen values before its
// partial enters a tree (cross-lane for rows, cross-wave / cross-workgroup for columns).
#include "lg_common.hpp"
#include <mutex>

namespace lg {

constexpr int kRThreads = 256;
constexpr int kRWaves = kRThreads / kWave;
constexpr int64_t kWideRowsBelow = 768;   // fewer rows than this (three per CU), each at least 32768 long: 1024-lane workgroups

typedef float f32x4 __attribute__((ext_vector_type(4)));

// 128-bit streaming load: the reductions touch every input element exactly once, so the lines are
// marked non-temporal (measured +10 % read bandwidth over plain loads on this part).
__device__ __forceinline__ float4 load_stream4(const float* p) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

// out[i] = sum_j in[i,j].  One workgroup per row when rows are long (WG_PER_ROW), one wavefront
// per row otherwise.  Each lane owns 128-bit columns strided by the group width; four loads are
// in flight per lane before the adds.
// With P > 1 a "row" is one of P segments of a row of the matrix: R counts segments, segment
// v = (r, q) starts at in + r*ld + q*Cn and is Cn long except the last of a row, which ends at
// Ctot (long rows cut into pieces so that a handful of them fills the chip; the piece sums are
// added by a second pass over the R/P x P matrix of partial sums).
// NTH: 256 lanes per workgroup, or 1024 when there are only a few long rows (what one CU draws from
// memory grows with the loads it has in flight).
template <bool VEC, bool WG_PER_ROW, int NTH = kRThreads>
__global__ __launch_bounds__(NTH) void reduce_rows_kernel(
    const float* __restrict__ in, float* __restrict__ out,
    int64_t R, int64_t Cn, int64_t ld, int accumulate, int64_t P, int64_t Ctot) {
    constexpr int NW = NTH / kWave;
    __shared__ float part[NW];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t row = WG_PER_ROW ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * NW + wave;
    const int width = WG_PER_ROW ? NTH : kWave;
    const int pos = WG_PER_ROW ? (int)threadIdx.x : lane;
    float s = 0.f;
    if (row < R) {
        const float* p = in + row * ld;
        if (P > 1) {
            const int64_t r = row / P, q = row - r * P;
            p = in + r * ld + q * Cn;
            if (Ctot - q * Cn < Cn) Cn = Ctot - q * Cn;
        }
        if constexpr (VEC) {
            const int64_t n4 = Cn / 4;
            float4 a0 = make_float4(0, 0, 0, 0), a1 = a0, a2 = a0, a3 = a0;
            int64_t j = pos;
            for (; j + 3 * width < n4; j += 4 * width) {
                const float4 v0 = load_stream4(p + 4 * j);
                const float4 v1 = load_stream4(p + 4 * (j + width));
                const float4 v2 = load_stream4(p + 4 * (j + 2 * width));
                const float4 v3 = load_stream4(p + 4 * (j + 3 * width));
                a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
                a1.x += v1.x; a1.y += v1.y; a1.z += v1.z; a1.w += v1.w;
                a2.x += v2.x; a2.y += v2.y; a2.z += v2.z; a2.w += v2.w;
                a3.x += v3.x; a3.y += v3.y; a3.z += v3.z; a3.w += v3.w;
            }
            for (; j < n4; j += width) {
                const float4 v0 = load_stream4(p + 4 * j);
                a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
            }
            s = ((a0.x + a1.x) + (a2.x + a3.x)) + ((a0.y + a1.y) + (a2.y + a3.y)) +
                (((a0.z + a1.z) + (a2.z + a3.z)) + ((a0.w + a1.w) + (a2.w + a3.w)));
        } else {
            float b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
            int64_t j = pos;
            for (; j + 3 * width < Cn; j += 4 * width) {
                b0 += p[j]; b1 += p[j + width]; b2 += p[j + 2 * width]; b3 += p[j + 3 * width];
            }
            for (; j < Cn; j += width) b0 += p[j];
            s = (b0 + b1) + (b2 + b3);
        }
    }
    s = wave_sum(s);
    if constexpr (WG_PER_ROW) {
        if (lane == 0) part[wave] = s;
        __syncthreads();
        if (threadIdx.x == 0) {
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < NW; w += 4) tot += (part[w] + part[w + 1]) + (part[w + 2] + part[w + 3]);
            if (accumulate) tot += out[row];
            out[row] = tot;
        }
    } else {
        if (lane == 0 && row < R) {
            if (accumulate) s += out[row];
            out[row] = s;
        }
    }
}

// Short rows (at most 64 accesses per row): a wavefront holds 64 / L rows at once, L = lanes per row
// (a power of two), and U batches of rows in flight, so no lane idles and each lane has U loads
// outstanding.  The row sum is a butterfly over the L lanes of a row.
template <bool VEC>
__global__ __launch_bounds__(kRThreads) void reduce_rows_short_kernel(
    const float* __restrict__ in, float* __restrict__ out,
    int64_t R, int64_t Cn, int64_t ld, int accumulate, int L) {
    constexpr int W = VEC ? 4 : 1;
    constexpr int U = 4;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int G = kWave / L;                        // rows per wavefront per batch
    const int sub = lane % L, rg = lane / L;
    const int64_t nw = Cn / W;                      // accesses per row (<= L)
    const int64_t row0 = ((int64_t)blockIdx.x * kRWaves + wave) * (G * U) + rg;
    float s[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t row = row0 + (int64_t)G * u;
        s[u] = 0.f;
        if (row < R && sub < nw) {
            const float* p = in + row * ld + W * sub;
            if constexpr (VEC) {
                const float4 v = load_stream4(p);
                s[u] = (v.x + v.y) + (v.z + v.w);
            } else {
                s[u] = *p;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float t = s[u];
        for (int off = L / 2; off > 0; off >>= 1) t += __shfl_xor(t, off, kWave);
        const int64_t row = row0 + (int64_t)G * u;
        if (sub == 0 && row < R) {
            if (accumulate) t += out[row];
            out[row] = t;
        }
    }
}

constexpr int kCRowsPerWave = 64;   // fewest rows a workgroup takes (16 per wavefront of a 4-wave workgroup)
constexpr int kCMaxSplit = 1024;

// Stage 1 of out[j] = sum_i in[i,j]: workgroup (bx, by) sums rows [by*rows_per_wg, ...) of the
// 64*W columns starting at bx*64*W.  Each lane owns W adjacent columns; the NTH/64 wavefronts take
// interleaved rows and are combined through LDS.  dst is the partial buffer (row by of width
// ldp) or the final output when the row range is not split.  NTH = 1024 for tall inputs (measured
// on 4096 x 16384: 16 waves x 512 rows per workgroup 45 us, 4 waves x 256 rows 50 us, combine included).
template <bool VEC, int NTH>
__global__ __launch_bounds__(NTH) void reduce_cols_kernel(
    const float* __restrict__ in, float* __restrict__ dst,
    int64_t R, int64_t Cn, int64_t ld, int64_t rows_per_wg, int64_t ldp, int final_accumulate) {
    constexpr int W = VEC ? 4 : 1;
    constexpr int NW = NTH / kWave;
    __shared__ float part[NW][kWave * W];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t col = ((int64_t)blockIdx.x * kWave + lane) * W;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_wg;
    const int64_t r1 = (r0 + rows_per_wg < R) ? r0 + rows_per_wg : R;
    float acc[2][W];
#pragma unroll
    for (int w = 0; w < W; ++w) acc[0][w] = acc[1][w] = 0.f;
    if (col < Cn) {
        const float* p = in + col;
        int64_t r = r0 + wave;
        if constexpr (VEC) {
            constexpr int U = 8;                     // rows in flight per lane
            for (; r + (U - 1) * NW < r1; r += U * NW) {
                float4 v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = load_stream4(p + (r + u * NW) * ld);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    acc[u & 1][0] += v[u].x; acc[u & 1][1] += v[u].y; acc[u & 1][2] += v[u].z; acc[u & 1][3] += v[u].w;
                }
            }
            for (; r < r1; r += NW) {
                const float4 v0 = load_stream4(p + r * ld);
                acc[0][0] += v0.x; acc[0][1] += v0.y; acc[0][2] += v0.z; acc[0][3] += v0.w;
            }
        } else {
            for (; r + NW < r1; r += 2 * NW) {
                acc[0][0] += p[r * ld];
                acc[1][0] += p[(r + NW) * ld];
            }
            for (; r < r1; r += NW) acc[0][0] += p[r * ld];
        }
    }
#pragma unroll
    for (int w = 0; w < W; ++w) part[wave][lane * W + w] = acc[0][w] + acc[1][w];
    __syncthreads();
    for (int c = threadIdx.x; c < kWave * W; c += NTH) {
        const int64_t gc = (int64_t)blockIdx.x * kWave * W + c;
        if (gc < Cn) {
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < NW; w += 4) tot += (part[w][c] + part[w + 1][c]) + (part[w + 2][c] + part[w + 3][c]);
            float* o = dst + (int64_t)blockIdx.y * ldp + gc;
            if (final_accumulate) tot += *o;
            *o = tot;
        }
    }
}

// Stage 1 for narrow inputs (at most 32 accesses per row): L lanes (a power of two) cover a row, so
// a wavefront reads 64 / L rows per access and no lane idles; the row groups of a wavefront are
// summed by a butterfly, the wavefronts through LDS as above.  One column strip (blockIdx.x = 0).
template <bool VEC, int NTH>
__global__ __launch_bounds__(NTH) void reduce_cols_narrow_kernel(
    const float* __restrict__ in, float* __restrict__ dst,
    int64_t R, int64_t Cn, int64_t ld, int64_t rows_per_wg, int64_t ldp, int final_accumulate, int L) {
    constexpr int W = VEC ? 4 : 1;
    constexpr int NW = NTH / kWave;
    constexpr int U = 8;                            // rows in flight per lane
    __shared__ float part[NW][32 * W];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int G = kWave / L;
    const int cq = lane % L, rg = lane / L;
    const int64_t col = (int64_t)cq * W;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_wg;
    const int64_t r1 = (r0 + rows_per_wg < R) ? r0 + rows_per_wg : R;
    const int64_t step = (int64_t)NW * G;           // rows between a lane's successive accesses
    float acc[2][W];
#pragma unroll
    for (int w = 0; w < W; ++w) acc[0][w] = acc[1][w] = 0.f;
    if (col < Cn) {
        const float* p = in + col;
        int64_t r = r0 + (int64_t)wave * G + rg;
        for (; r + (U - 1) * step < r1; r += U * step) {
            float v[U][W];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (VEC) {
                    const float4 q = load_stream4(p + (r + u * step) * ld);
                    v[u][0] = q.x; v[u][1] = q.y; v[u][2] = q.z; v[u][3] = q.w;
                } else {
                    v[u][0] = p[(r + u * step) * ld];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int w = 0; w < W; ++w) acc[u & 1][w] += v[u][w];
        }
        for (; r < r1; r += step) {
            if constexpr (VEC) {
                const float4 q = load_stream4(p + r * ld);
                acc[0][0] += q.x; acc[0][1] += q.y; acc[0][2] += q.z; acc[0][3] += q.w;
            } else {
                acc[0][0] += p[r * ld];
            }
        }
    }
#pragma unroll
    for (int w = 0; w < W; ++w) {
        float t = acc[0][w] + acc[1][w];
        for (int off = L; off < kWave; off <<= 1) t += __shfl_xor(t, off, kWave);
        if (rg == 0) part[wave][cq * W + w] = t;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < L * W; c += NTH) {
        if (c < Cn) {
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < NW; w += 4) tot += (part[w][c] + part[w + 1][c]) + (part[w + 2][c] + part[w + 3][c]);
            float* o = dst + (int64_t)blockIdx.y * ldp + c;
            if (final_accumulate) tot += *o;
            *o = tot;
        }
    }
}

// Stage 2 for many partial rows (tall narrow inputs): out[j] (+)= sum_s partial[s][j], in a fixed
// order.  A workgroup owns 64 columns; its NSL split-lanes per column each add every NSL-th partial
// (four running sums), then a tree in LDS adds the split-lanes.
template <int NSL>
__global__ __launch_bounds__(64 * NSL) void reduce_cols_combine_kernel(
    const float* __restrict__ partial, float* __restrict__ out,
    int64_t Cn, int64_t ldp, int splits, int accumulate) {
    __shared__ float part[NSL][64];
    const int c = threadIdx.x % 64, sl = threadIdx.x / 64;
    const int64_t j = (int64_t)blockIdx.x * 64 + c;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    if (j < Cn) {
        int sp = sl;
        for (; sp + 3 * NSL < splits; sp += 4 * NSL) {
            a0 += partial[(int64_t)sp * ldp + j];
            a1 += partial[(int64_t)(sp + NSL) * ldp + j];
            a2 += partial[(int64_t)(sp + 2 * NSL) * ldp + j];
            a3 += partial[(int64_t)(sp + 3 * NSL) * ldp + j];
        }
        for (; sp < splits; sp += NSL) a0 += partial[(int64_t)sp * ldp + j];
    }
    part[sl][c] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    for (int half = NSL / 2; half > 0; half /= 2) {
        if (sl < half) part[sl][c] += part[sl + half][c];
        __syncthreads();
    }
    if (sl == 0 && j < Cn) {
        float tot = part[0][c];
        if (accumulate) tot += out[j];
        out[j] = tot;
    }
}

// Stage 2 for a handful of partial rows (the tall benchmark shape has 8): one lane per column, every
// partial requested before the first add, no LDS and no barrier -- the kernel is one memory round
// trip long (measured behind a 256 MiB read: 1.3 us per launch against 4.5 for the kernel above).
// Fixed order: a balanced tree over ascending row chunks.
template <int MAXS>
__global__ __launch_bounds__(256) void reduce_cols_combine_flat_kernel(
    const float* __restrict__ partial, float* __restrict__ out, int64_t Cn, int64_t ldp, int splits, int accumulate) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= Cn) return;
    float v[MAXS];
#pragma unroll
    for (int sp = 0; sp < MAXS; ++sp) v[sp] = sp < splits ? partial[(int64_t)sp * ldp + j] : 0.f;
    float tot = 0.f;
#pragma unroll
    for (int sp = 0; sp < MAXS; sp += 4) tot += (v[sp] + v[sp + 1]) + (v[sp + 2] + v[sp + 3]);
    if (accumulate) tot += out[j];
    out[j] = tot;
}

__global__ void fill_zero_kernel(float* out, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = 0.f;
}

struct ColPlan { int64_t splits, rows_per_wg, ldp; bool big; };

static ColPlan plan_cols(int64_t R, int64_t Cn) {
    ColPlan p;
    const int64_t strips = cdiv(Cn, 256);          // column strips of the 128-bit kernel
    // 16-wave workgroups over 512 rows each are the fastest shape (measured), as long as they still
    // make more than a hundred workgroups; otherwise 4-wave workgroups, about 2048 of them, over at
    // least 64 rows each -- 256 once the strips alone give every CU a workgroup (a second launch to
    // combine the chunks then costs more than the extra parallelism returns).
    p.big = R >= 2048 && strips * cdiv(R, 512) >= 128;
    // A small input is one launch: a 16-wave workgroup keeps 16 x 8 rows in flight (64 / L times that
    // when L <= 32 lanes cover a row, counting one float per lane as the unaligned case does), and up
    // to four such round trips cost less than a second launch that adds the chunks (measured back to
    // back: 100 x 4098 9.5 -> one launch).
    int64_t in_flight = 16 * 8;
    if (Cn <= 32) {
        int64_t L = 1;
        while (L < Cn) L *= 2;
        in_flight *= kWave / L;
    }
    if (R <= 4 * in_flight && R * Cn <= ((int64_t)1 << 20)) {    // up to 4 MB: beyond that the chunks are worth their launch
        p.big = R >= 64;
        p.splits = 1;
        p.rows_per_wg = R;
        p.ldp = cdiv(Cn, 64) * 64;
        return p;
    }
    int64_t rows;
    if (p.big) {
        rows = 512;
    } else {
        const int64_t want = cdiv(2048, strips);   // row chunks wanted
        const int64_t least = strips >= 256 ? (int64_t)kCRowsPerWave * kRWaves : kCRowsPerWave;
        rows = cdiv(R, want);
        if (rows < least) rows = least;
    }
    int64_t splits = cdiv(R, rows);
    if (splits > kCMaxSplit) splits = kCMaxSplit;
    if (splits < 1) splits = 1;
    p.rows_per_wg = cdiv(R, splits);
    p.splits = cdiv(R, p.rows_per_wg);
    p.ldp = cdiv(Cn, 64) * 64;
    return p;
}

}  // namespace lg

namespace lg {

// How lg_reduce_rows_ws cuts long rows: P pieces per row, each `len` long (a multiple of 1024
// floats, one pass of a workgroup's 128-bit accesses), once the rows alone cannot fill the chip.
struct RowPlan { int64_t P, len; };
static RowPlan plan_rows(int64_t R, int64_t Cn) {
    RowPlan pl{1, Cn};
    if (R >= 512 || Cn < 32768) return pl;                     // enough rows, or rows too short to cut
    int64_t P = 2048 / R;                                      // ~8 workgroups per CU in all
    if (P > Cn / 8192) P = Cn / 8192;                          // pieces of at least 8192 floats
    if (P < 2) return pl;
    pl.len = cdiv(cdiv(Cn, P), 1024) * 1024;
    pl.P = cdiv(Cn, pl.len);
    if (pl.P < 2) return RowPlan{1, Cn};
    return pl;
}

static int reduce_rows_impl(const float* in, float* out, int64_t R, int64_t Cn, int64_t ld,
                            int accumulate, hipStream_t s);

}  // namespace lg

extern "C" size_t lg_reduce_rows_workspace_bytes(int64_t R, int64_t Cn) {
    using namespace lg;
    if (R <= 0 || Cn <= 0) return 0;
    const RowPlan pl = plan_rows(R, Cn);
    return pl.P > 1 ? (size_t)(R * pl.P) * sizeof(float) : 0;
}

extern "C" int lg_reduce_rows_ws(const float* in, float* out, int64_t R, int64_t Cn, int64_t ld,
                                 int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace lg;
    if (R < 0 || Cn < 0 || ld < Cn) return LG_ERR_INVALID_ARG;
    if (R == 0) return LG_OK;
    if (!out || (Cn > 0 && !in)) return LG_ERR_INVALID_ARG;
    if (Cn > 0 && overlaps(in, ((R - 1) * ld + Cn) * 4, out, R * 4)) return LG_ERR_INVALID_ARG;
    hipStream_t s = begin_call(stream);
    const RowPlan pl = plan_rows(R, Cn);
    if (pl.P <= 1) return reduce_rows_impl(in, out, R, Cn, ld, accumulate, s);
    const size_t need = (size_t)(R * pl.P) * sizeof(float);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return LG_ERR_WORKSPACE;
    if (overlaps(workspace, (int64_t)need, out, R * 4) ||
        overlaps(workspace, (int64_t)need, in, ((R - 1) * ld + Cn) * 4))
        return LG_ERR_INVALID_ARG;
    float* partial = static_cast<float*>(workspace);
    const bool vec = (Cn % 4 == 0) && (ld % 4 == 0) && aligned16(in);
    const dim3 g((unsigned)(R * pl.P)), b(kRThreads);          // R < 512 and P <= 2048 / R
    if (vec) hipLaunchKernelGGL((reduce_rows_kernel<true, true>), g, b, 0, s, in, partial, R * pl.P, pl.len, ld, 0, pl.P, Cn);
    else     hipLaunchKernelGGL((reduce_rows_kernel<false, true>), g, b, 0, s, in, partial, R * pl.P, pl.len, ld, 0, pl.P, Cn);
    if (launch_status() != LG_OK) return LG_ERR_RUNTIME;
    return reduce_rows_impl(partial, out, R, pl.P, pl.P, accumulate, s);
}

extern "C" int lg_reduce_rows(const float* in, float* out, int64_t R, int64_t Cn, int64_t ld,
                              int accumulate, void* stream) {
    using namespace lg;
    if (R < 0 || Cn < 0 || ld < Cn) return LG_ERR_INVALID_ARG;
    if (R == 0) return LG_OK;
    if (!out || (Cn > 0 && !in)) return LG_ERR_INVALID_ARG;
    if (Cn > 0 && overlaps(in, ((R - 1) * ld + Cn) * 4, out, R * 4)) return LG_ERR_INVALID_ARG;
    return reduce_rows_impl(in, out, R, Cn, ld, accumulate, begin_call(stream));
}

namespace lg {

static int reduce_rows_impl(const float* in, float* out, int64_t R, int64_t Cn, int64_t ld,
                            int accumulate, hipStream_t s) {
    const bool vec = Cn > 0 && (Cn % 4 == 0) && (ld % 4 == 0) && aligned16(in);
    const int64_t accesses = vec ? Cn / 4 : Cn;     // per row
    if (accesses >= 1 && accesses <= kWave) {
        int L = 1;
        while (L < accesses) L *= 2;
        const int64_t rows_per_wg = (int64_t)kRWaves * (kWave / L) * 4;
        const int64_t nb = cdiv(R, rows_per_wg);
        if (nb > kMaxGrid) return LG_ERR_UNSUPPORTED;
        if (vec) hipLaunchKernelGGL(reduce_rows_short_kernel<true>, dim3((unsigned)nb), dim3(kRThreads), 0, s, in, out, R, Cn, ld, accumulate, L);
        else     hipLaunchKernelGGL(reduce_rows_short_kernel<false>, dim3((unsigned)nb), dim3(kRThreads), 0, s, in, out, R, Cn, ld, accumulate, L);
        return launch_status();
    }
    const bool wg_per_row = Cn >= 4096;
    const int64_t blocks = wg_per_row ? R : cdiv(R, kRWaves);
    if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
    const dim3 g((unsigned)blocks), b(kRThreads);
    // a few long rows: 16 wavefronts per row instead of 4 (3 x 1 000 000: 184 -> 32 us; 256 x 131072: 35 -> 20 us)
    // ... and rows that 1024 lanes cover in whole trips of four accesses each: the row is requested in one
    // go and the workgroup retires (4096 x 16384, cold, back to back: 42.7 -> 41.4 us)
    if (wg_per_row && ((R < kWideRowsBelow && Cn >= 32768) || (Cn >= 16384 && Cn % 4096 == 0))) {
        if (vec) hipLaunchKernelGGL((reduce_rows_kernel<true, true, 1024>), g, dim3(1024), 0, s, in, out, R, Cn, ld, accumulate, (int64_t)1, Cn);
        else     hipLaunchKernelGGL((reduce_rows_kernel<false, true, 1024>), g, dim3(1024), 0, s, in, out, R, Cn, ld, accumulate, (int64_t)1, Cn);
        return launch_status();
    }
    if (vec && wg_per_row)       hipLaunchKernelGGL((reduce_rows_kernel<true, true>), g, b, 0, s, in, out, R, Cn, ld, accumulate, (int64_t)1, Cn);
    else if (vec)                hipLaunchKernelGGL((reduce_rows_kernel<true, false>), g, b, 0, s, in, out, R, Cn, ld, accumulate, (int64_t)1, Cn);
    else if (wg_per_row)         hipLaunchKernelGGL((reduce_rows_kernel<false, true>), g, b, 0, s, in, out, R, Cn, ld, accumulate, (int64_t)1, Cn);
    else                         hipLaunchKernelGGL((reduce_rows_kernel<false, false>), g, b, 0, s, in, out, R, Cn, ld, accumulate, (int64_t)1, Cn);
    return launch_status();
}

}  // namespace lg

extern "C" size_t lg_reduce_cols_workspace_bytes(int64_t R, int64_t Cn) {
    using namespace lg;
    if (R <= 0 || Cn <= 0) return 0;
    const ColPlan p = plan_cols(R, Cn);
    return p.splits > 1 ? (size_t)(p.splits * p.ldp) * sizeof(float) : 0;
}

namespace lg {

// Both column-reduction entry points: argument checks, plan, stage 1 and (when the rows are split)
// stage 2.  `partial` is the scratch for the chunk sums; the caller has checked that it is there,
// large enough and clear of the operands whenever the plan splits the rows.
static int reduce_cols_impl(const float* in, float* out, int64_t R, int64_t Cn, int64_t ld,
                            int accumulate, float* partial, const ColPlan& p, hipStream_t s) {
    const bool vec = (Cn % 4 == 0) && (ld % 4 == 0) && aligned16(in);
    const int64_t bx = cdiv(Cn, vec ? 256 : 64);
    if (bx > kMaxGrid || cdiv(Cn, 64) > kMaxGrid || p.splits > 65535) return LG_ERR_UNSUPPORTED;
    const dim3 g((unsigned)bx, (unsigned)p.splits), b(kRThreads), b16(1024);
    float* dst = p.splits > 1 ? partial : out;
    const int64_t ldp = p.splits > 1 ? p.ldp : 0;
    const int facc = p.splits > 1 ? 0 : accumulate;
    const int64_t accesses = vec ? Cn / 4 : Cn;     // per row
    if (accesses <= 32) {                           // narrow: several rows per wavefront access
        int L = 1;
        while (L < accesses) L *= 2;
        const dim3 gn(1, (unsigned)p.splits);
        if (vec && p.big) hipLaunchKernelGGL((reduce_cols_narrow_kernel<true, 1024>), gn, b16, 0, s, in, dst, R, Cn, ld, p.rows_per_wg, ldp, facc, L);
        else if (vec)     hipLaunchKernelGGL((reduce_cols_narrow_kernel<true, 256>), gn, b, 0, s, in, dst, R, Cn, ld, p.rows_per_wg, ldp, facc, L);
        else if (p.big)   hipLaunchKernelGGL((reduce_cols_narrow_kernel<false, 1024>), gn, b16, 0, s, in, dst, R, Cn, ld, p.rows_per_wg, ldp, facc, L);
        else              hipLaunchKernelGGL((reduce_cols_narrow_kernel<false, 256>), gn, b, 0, s, in, dst, R, Cn, ld, p.rows_per_wg, ldp, facc, L);
    } else
    if (vec && p.big) hipLaunchKernelGGL((reduce_cols_kernel<true, 1024>), g, b16, 0, s, in, dst, R, Cn, ld, p.rows_per_wg, ldp, facc);
    else if (vec)     hipLaunchKernelGGL((reduce_cols_kernel<true, 256>), g, b, 0, s, in, dst, R, Cn, ld, p.rows_per_wg, ldp, facc);
    else if (p.big)   hipLaunchKernelGGL((reduce_cols_kernel<false, 1024>), g, b16, 0, s, in, dst, R, Cn, ld, p.rows_per_wg, ldp, facc);
    else              hipLaunchKernelGGL((reduce_cols_kernel<false, 256>), g, b, 0, s, in, dst, R, Cn, ld, p.rows_per_wg, ldp, facc);
    if (launch_status() != LG_OK) return LG_ERR_RUNTIME;
    if (p.splits > 1) {
        const dim3 gc((unsigned)cdiv(Cn, 64));
        if (p.splits <= 8)
            hipLaunchKernelGGL(reduce_cols_combine_flat_kernel<8>, dim3((unsigned)cdiv(Cn, 256)), dim3(256), 0, s,
                               partial, out, Cn, p.ldp, (int)p.splits, accumulate);
        else if (p.splits <= 16)
            hipLaunchKernelGGL(reduce_cols_combine_flat_kernel<16>, dim3((unsigned)cdiv(Cn, 256)), dim3(256), 0, s,
                               partial, out, Cn, p.ldp, (int)p.splits, accumulate);
        else
            hipLaunchKernelGGL(reduce_cols_combine_kernel<16>, gc, dim3(1024), 0, s,
                               partial, out, Cn, p.ldp, (int)p.splits, accumulate);
        return launch_status();
    }
    return LG_OK;
}

// Argument checks shared by the column-reduction entry points; *done is set when the call is
// finished (an error, nothing to do, or the zero-row case, which is handled here).
static int reduce_cols_check(const float* in, float* out, int64_t R, int64_t Cn, int64_t ld,
                             int accumulate, hipStream_t s, bool* done) {
    *done = true;
    if (R < 0 || Cn < 0 || ld < Cn) return LG_ERR_INVALID_ARG;
    if (Cn == 0) return LG_OK;
    if (!out || (R > 0 && !in)) return LG_ERR_INVALID_ARG;
    if (R > 0 && overlaps(in, ((R - 1) * ld + Cn) * 4, out, Cn * 4)) return LG_ERR_INVALID_ARG;
    if (R == 0) {
        if (!accumulate) {
            const int64_t blocks = cdiv(Cn, 256);
            if (blocks > kMaxGrid) return LG_ERR_UNSUPPORTED;
            hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, out, Cn);
            return launch_status();
        }
        return LG_OK;
    }
    *done = false;
    return LG_OK;
}

}  // namespace lg

extern "C" int lg_reduce_cols(const float* in, float* out, int64_t R, int64_t Cn, int64_t ld,
                              int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace lg;
    hipStream_t s = begin_call(stream);
    bool done;
    const int rc = reduce_cols_check(in, out, R, Cn, ld, accumulate, s, &done);
    if (done) return rc;
    const ColPlan p = plan_cols(R, Cn);
    const size_t need = p.splits > 1 ? (size_t)(p.splits * p.ldp) * sizeof(float) : 0;
    if (need > 0) {
        if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
            return LG_ERR_WORKSPACE;
        if (overlaps(workspace, (int64_t)need, out, Cn * 4) ||
            overlaps(workspace, (int64_t)need, in, ((R - 1) * ld + Cn) * 4))
            return LG_ERR_INVALID_ARG;
    }
    return reduce_cols_impl(in, out, R, Cn, ld, accumulate, static_cast<float*>(workspace), p, s);
}

// ---- lg_reduce_cols for callers that cannot allocate ---------------------------------------------
// The chunk sums go to a fixed array in device memory that belongs to the library instead of a
// workspace the caller brings.  Every GPU the library runs on holds its own copy of the array (at
// its own address) until the process ends; the array's name below is only the host-side handle of
// the symbol, so host code asks the runtime once per device for the device address and passes that
// to the kernels.
namespace lg {

constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// device address of `scratch` on the current device, looked up on the first call there
static int static_scratch(float** ptr) {
    static std::mutex mu;
    static void* addr[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LG_ERR_RUNTIME;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LG_ERR_RUNTIME;
        addr[dev] = p;
    }
    *ptr = static_cast<float*>(addr[dev]);
    return LG_OK;
}

}  // namespace lg

extern "C" int lg_reduce_cols_static(const float* in, float* out, int64_t R, int64_t Cn, int64_t ld,
                                     int accumulate, void* stream) {
    using namespace lg;
    hipStream_t s = begin_call(stream);
    bool done;
    const int rc = reduce_cols_check(in, out, R, Cn, ld, accumulate, s, &done);
    if (done) return rc;
    const ColPlan p = plan_cols(R, Cn);
    const size_t need = p.splits > 1 ? (size_t)(p.splits * p.ldp) * sizeof(float) : 0;
    if (need > kStaticScratchBytes) return LG_ERR_UNSUPPORTED;
    float* partial = nullptr;
    if (need > 0) {
        const int sc = static_scratch(&partial);
        if (sc != LG_OK) return sc;
    }
    return reduce_cols_impl(in, out, R, Cn, ld, accumulate, partial, p, s);
}
