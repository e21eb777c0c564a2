// Shared device/host helpers for the gfx950 kernels of the TWN hot path.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "twn.h"

namespace twn {

constexpr int kWave = 64;

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline int32_t launch_status() {
    return hipGetLastError() == hipSuccess ? TWN_OK : TWN_ERR_HIP;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Environment override for launch-shape sweeps (0 / unset = built-in choice).
int env_int(const char* name, int fallback);

// ---- wave / block reductions in a fixed order (bit-identical run to run) ----
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Block-wide sum for blocks of up to 16 waves; every thread gets the result.
// `scratch` must hold 16 values and is reusable after the call returns.
template <typename T>
__device__ __forceinline__ T block_sum(T v, T* scratch) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int nwaves = (blockDim.x + kWave - 1) / kWave;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    T total = scratch[0];
    for (int w = 1; w < nwaves; ++w) total += scratch[w];
    return total;
}

// float -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// Two floats -> two bf16 in one register (low half = a), round to nearest even: one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// 2-bit field of the packed format: bit0 = non-zero, bit1 = negative.
__device__ __forceinline__ uint32_t code_field(float w, float delta) {
    const uint32_t nz = fabsf(w) > delta ? 1u : 0u;
    const uint32_t neg = (w < 0.0f) ? nz : 0u;
    return nz | (neg << 1);
}

}  // namespace twn
