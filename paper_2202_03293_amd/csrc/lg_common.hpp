// Shared host/device helpers of liblg (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <type_traits>
#include "lg.h"

namespace lg {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kXcds = 8;           // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin
constexpr int64_t kMaxGrid = 0x7FFFFFFF;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// [a, a+na) and [b, b+nb) byte ranges overlap?
inline bool overlaps(const void* a, int64_t na, const void* b, int64_t nb) {
    if (na <= 0 || nb <= 0) return false;
    uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + static_cast<uintptr_t>(nb) && b0 < a0 + static_cast<uintptr_t>(na);
}

// Raise a kernel's dynamic-LDS limit once per device (the attribute belongs to the kernel as loaded
// on one device).  `done` is the caller's per-kernel table of kMaxDevices flags; two host threads that
// meet on a kernel's first use both set the attribute (to the same value), which is harmless.
constexpr int kMaxDevices = 64;
using DeviceFlags = std::atomic<bool>[kMaxDevices];
inline void allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<bool>* done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = -1;
    if (dev >= 0 && done[dev].load(std::memory_order_acquire)) return;
    (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (dev >= 0) done[dev].store(true, std::memory_order_release);
}

// The runtime keeps one "last error" per host thread, shared with every other user of HIP in the
// process.  An entry point that launches takes its stream through begin_call(), which clears
// whatever an earlier caller left there, so that launch_status() after a launch reports this
// library's launches only.
inline hipStream_t begin_call(void* stream) {
    (void)hipGetLastError();
    return static_cast<hipStream_t>(stream);
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? LG_OK : LG_ERR_RUNTIME; }

// Workgroups are handed to the 8 XCDs round-robin (hardware id i runs on XCD i % 8) and each XCD
// has a private L2.  This turns a hardware workgroup id into a logical one such that each XCD works
// on one contiguous range of logical ids, so neighbouring tiles share an L2.
__device__ __forceinline__ unsigned xcd_contiguous_id(unsigned bid, unsigned nblocks) {
    const unsigned per = nblocks / kXcds, rem = nblocks % kXcds;
    const unsigned x = bid % kXcds, l = bid / kXcds;
    return x * per + (x < rem ? x : rem) + l;
}

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
                 :: "s"(lds), "v"(voff), "s"(base) : "memory", "m0");
}

// The same with 4 bytes per lane (lane l's word lands at lds + 4*l): for operands whose rows are not
// 16-byte aligned.  Four times the instructions for the same bytes.
__device__ __forceinline__ void dma4(const void* base, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(lds), "v"(voff), "s"(base) : "memory", "m0");
}

// Wait until at most N of this wave's global->LDS transfers are still in flight.
template <int N>
__device__ __forceinline__ void dma_wait() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// A wave-uniform 64-bit value moved into scalar registers (64-bit divisions leave theirs in vector
// registers even when every lane holds the same number).
__device__ __forceinline__ int64_t to_scalar(int64_t v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// f(integral_constant<int, B>), ..., f(integral_constant<int, E - 1>): a loop whose index is a
// compile-time constant in the body (s_waitcnt takes its count as an immediate).
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

}  // namespace lg
