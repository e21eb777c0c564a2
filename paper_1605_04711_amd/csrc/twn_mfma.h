// Device helpers shared by the MFMA contraction kernels (gfx950).
#pragma once

#include "twn_common.h"

namespace twn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Exact unsigned division of numerators below 2^31 by a runtime constant.
struct FastDivU {
    uint32_t mul, shift, one;   // one = all ones when d == 1 (then mul = 0 and the quotient is n itself)
};

static inline FastDivU make_fastdiv_u(uint32_t d) {
    FastDivU f{0, 0, 0xFFFFFFFFu};
    if (d <= 1) return f;
    f.one = 0;
    uint32_t l = 0;
    while ((1u << l) < d) ++l;
    const uint32_t s = 31 + l;
    f.mul = static_cast<uint32_t>(((1ULL << s) + d - 1) / d);
    f.shift = s - 32;
    return f;
}

__device__ __forceinline__ uint32_t fdiv_u(uint32_t n, const FastDivU& f) {
    return (__umulhi(n, f.mul) >> f.shift) | (n & f.one);
}

// s_waitcnt immediate that waits only for vmcnt <= n (gfx9 encoding).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// One direct global -> LDS load of 16 bytes per lane: lane j of the wave writes LDS at lds_dst + 16*j
// (lds_dst is wave-uniform); counted by vmcnt.
__device__ __forceinline__ void dma16(const void* gsrc, void* lds_dst) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                     (__attribute__((address_space(3))) void*)lds_dst, 16, 0, 0);
}

// The same through a raw buffer descriptor: address = base + voffset (per lane) + soffset (wave-uniform, so
// advancing along K costs no vector instruction); a lane whose voffset is at or beyond the descriptor's
// size reads zeros, which replaces the select against a zero block for rows and taps outside the tensor.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, static_cast<int>(bytes), 0x00020000);
}
__device__ __forceinline__ void buf_dma16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voffset, uint32_t soffset, void* lds_dst) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)lds_dst, 16,
                                             static_cast<int>(voffset), static_cast<int>(soffset), 0, 0);
}
constexpr uint32_t kBufOutside = 0x80000000u;   // voffset of a lane that must read zeros (tensors stay below 2 GiB)
// Cache policy of the output stores of the persistent contraction kernels (buffer-store auxiliary bit 4 = sc1): the line is
// written through to memory when it is stored instead of staying dirty in the XCD's L2 until the release at the end
// of the kernel, which would write a layer's whole output back in one burst while the next kernel waits (ResNet-18
// b64 forward: 0.452 -> 0.440 ms).  The data still stays in the cache for the next layer (the non-temporal hint
// instead makes single layers faster and the chain slower, because the consumer then reads from memory).
constexpr int kStoreThrough = 16;
// The same policy for a 16-byte store through a plain pointer (outputs addressed with 64-bit offsets).
__device__ __forceinline__ void store16_through(void* p, const u32x4& v) {
    // the wait states ride in the same statement: the compiler cannot see that this is a store of more than 8 bytes, so
    // it would not keep the next instruction from overwriting the data registers while they are still being read
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}

}  // namespace twn
