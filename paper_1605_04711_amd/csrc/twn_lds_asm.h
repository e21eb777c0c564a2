// Inline-assembly LDS reads with hand-placed waits, and compile-time loop helpers, shared by the
// direct-to-LDS contraction kernels (gfx950).
#pragma once

#include <type_traits>
#include <utility>

#include "twn_mfma.h"

namespace twn {

// LDS reads of the main loop are written as inline assembly with hand-placed s_waitcnt lgkmcnt(n): the
// compiler's own wait insertion falls back to lgkmcnt(0) in this loop, which also waits for the reads
// issued one MFMA step ahead and so exposes the whole LDS latency at every step.  LDS operations
// complete in issue order, so "at most n outstanding" is exact.  A value read this way may only be
// consumed after lds_wait<n>() followed by lds_ready() on its registers.
template <int OFFSET>
__device__ __forceinline__ void lds_read128(u32x4& d, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFFSET));
}
template <int OFFSET>
__device__ __forceinline__ void lds_read64(u32x2& d, uint32_t addr) {
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFFSET));
}
// N reads (N <= 8) at addr, addr + STRIDE, ...
template <int N, int STRIDE>
__device__ __forceinline__ void lds_read128_n(u32x4* d, uint32_t addr) {
    static_assert(N >= 1 && N <= 8 && (N - 1) * STRIDE < 65536, "immediate offsets");
    lds_read128<0>(d[0], addr);
    if constexpr (N > 1) lds_read128<STRIDE>(d[1], addr);
    if constexpr (N > 2) lds_read128<2 * STRIDE>(d[2], addr);
    if constexpr (N > 3) lds_read128<3 * STRIDE>(d[3], addr);
    if constexpr (N > 4) lds_read128<4 * STRIDE>(d[4], addr);
    if constexpr (N > 5) lds_read128<5 * STRIDE>(d[5], addr);
    if constexpr (N > 6) lds_read128<6 * STRIDE>(d[6], addr);
    if constexpr (N > 7) lds_read128<7 * STRIDE>(d[7], addr);
}
template <int N, int STRIDE>
__device__ __forceinline__ void lds_read64_n(u32x2* d, uint32_t addr) {
    static_assert(N >= 1 && N <= 4 && 3 * STRIDE < 65536, "immediate offsets");
    lds_read64<0>(d[0], addr);
    if constexpr (N > 1) lds_read64<STRIDE>(d[1], addr);
    if constexpr (N > 2) lds_read64<2 * STRIDE>(d[2], addr);
    if constexpr (N > 3) lds_read64<3 * STRIDE>(d[3], addr);
}
template <int N>
__device__ __forceinline__ void lds_wait() {
    static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N));
}
// ties the consumers of r[0..N) to the preceding lds_wait (volatile asm statements keep their order)
template <int N, class T>
__device__ __forceinline__ void lds_ready(T* r) {
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(r[i]));
}

// a constant the compiler keeps in a scalar register (it cannot fold it back into a literal operand)
template <int V>
__device__ __forceinline__ uint32_t sgpr_const() {
    uint32_t r;
    asm volatile("s_mov_b32 %0, %1" : "=s"(r) : "n"(V));
    return r;
}

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

}  // namespace twn
