// Output path of the persistent contraction kernels (Eq. 2 with the scaling factor of Eq. 5 applied after the
// additions; per-channel scale / shift, residual and ReLU of the following layers fused): one wave turns its
// MI x NI accumulator tiles into bf16 rows and writes them.
//
// The output path is bound by vector-ALU issue (every wave of the chip runs it at the same time), so it is
// written for few instructions per value: one FMA, half a convert (two values per v_cvt_pk_bf16_f32) and half
// an integer max (ReLU on the packed pair: a negative bf16 is a negative int16; rounding first and clamping
// afterwards gives the same bits as clamping first, rounding keeps the sign).  Addresses are buffer offsets:
// the per-lane part is fixed for the whole kernel, the tile and row-block part is wave-uniform and goes into
// the scalar offset, rows and columns outside the tensor get an offset beyond the descriptor (loads return
// zero, stores are dropped), and a tile that lies fully inside needs no bounds arithmetic at all.  Residual
// values of row block mi+1 are requested before row block mi is processed.
#pragma once

#include "twn_common.h"
#include "twn_mfma.h"

namespace twn {

typedef short s16x2 __attribute__((ext_vector_type(2)));

// Lane-fixed parts of the output addresses (bytes), set up once per kernel.
template <int EPI_CH>
struct TileStoreLane {
    static constexpr int LPR = EPI_CH / 8;            // lanes per staged row (16 bytes each)
    static constexpr int NIT = 32 * LPR / 64;         // store instructions per 32-row block
    static constexpr int RPI = 64 / LPR;              // rows per store instruction
    uint32_t res_off;                                 // row lrow, column lh*4 of a 32x32 accumulator tile
    uint32_t st_off[NIT];                             // row it*RPI + lane/LPR, column (lane%LPR)*8
    __device__ __forceinline__ void init(int lane, uint32_t ldyB) {
        res_off = static_cast<uint32_t>(lane & 31) * ldyB + static_cast<uint32_t>(lane >> 5) * 8u;
#pragma unroll
        for (int it = 0; it < NIT; ++it)
            st_off[it] = static_cast<uint32_t>(it * RPI + lane / LPR) * ldyB + static_cast<uint32_t>(lane % LPR) * 16u;
    }
};

// acc[mi][ni] element e of this lane: row mi*32 + (lane & 31), column ni*32 + (e>>2)*8 + (lane>>5)*4 + (e&3)
// of the wave's tile, whose first row / column in the output are m_first / n_first (wave-uniform).
// cmul / cadd: LDS, per column of the wave's tile.  stg: the wave's staging rows (32 rows of EPI_CH*2+16 bytes).
// ry / rr: descriptors of Y and of the residual (same layout; rr is only used when has_res).
// relu_floor: 0 with ReLU, 0x80008000 without (int16 minimum in both halves).
// FULL: the wave's tile lies inside the tensor (no bounds arithmetic).
template <int MI, int NI, int EPI_CH, bool FULL>
__device__ __forceinline__ void store_tile_bf16(const f32x16 (&acc)[MI][NI], const float* cmul, const float* cadd,
                                                unsigned char* stg, const TileStoreLane<EPI_CH>& L,
                                                __amdgpu_buffer_rsrc_t ry, __amdgpu_buffer_rsrc_t rr, bool has_res,
                                                uint32_t m_first, int n_first, uint32_t M, int NC, uint32_t ldyB,
                                                uint32_t relu_floor, int lane) {
    constexpr int EPI_ROW = EPI_CH * 2 + 16;
    constexpr int EPI_NI = EPI_CH / 32;
    constexpr int NIT = TileStoreLane<EPI_CH>::NIT, RPI = TileStoreLane<EPI_CH>::RPI, LPR = TileStoreLane<EPI_CH>::LPR;
    const int lrow = lane & 31, lh = lane >> 5;
    // rows and columns of the wave's tile that exist (wave-uniform)
    int rows_in = (M > m_first) ? static_cast<int>(M - m_first < 65536u ? M - m_first : 65536u) : 0;
    int cols_in = NC - n_first;
    // the edge path is rare: keep its bounds arithmetic inside it (nothing of it is worth holding in registers
    // across the main loop, which is what hoisting the tile-invariant parts would do)
    if (!FULL) asm volatile("" : "+s"(rows_in), "+s"(cols_in));
    const uint32_t tile_off = __builtin_amdgcn_readfirstlane(m_first * ldyB + static_cast<uint32_t>(n_first) * 2u);
    const s16x2 floor2 = __builtin_bit_cast(s16x2, relu_floor);

    // this lane's columns: multiplier and offset, held in registers for the whole tile when the accumulators
    // leave room for them (32 registers per 32 columns), else read from LDS for every row block
    constexpr bool HOIST = false;
    f32x4 mulv[HOIST ? NI : 1][4], addv[HOIST ? NI : 1][4];
    if constexpr (HOIST) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                mulv[ni][q4] = *reinterpret_cast<const f32x4*>(cmul + ni * 32 + q4 * 8 + lh * 4);
                addv[ni][q4] = *reinterpret_cast<const f32x4*>(cadd + ni * 32 + q4 * 8 + lh * 4);
            }
    }

    // residual values: requested one row block ahead into a second buffer, or (large accumulator tiles, where
    // registers are short) into the same buffer as soon as the current block's values are consumed
    constexpr int RES_BUF = (MI * NI >= 8) ? 1 : 2;
    u32x2 rres[RES_BUF][NI][4];
    auto res_load = [&](int mi, u32x2 (&dst)[NI][4]) __attribute__((always_inline)) {
        const uint32_t so = tile_off + static_cast<uint32_t>(mi * 32) * ldyB;
        const bool row_ok = FULL || (mi * 32 + lrow < rows_in);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                // the constant part of the column offset rides in the scalar offset: no per-lane variants
                const bool ok = FULL || (row_ok && ni * 32 + q4 * 8 + lh * 4 < cols_in);
                dst[ni][q4] = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(
                                                            rr, ok ? L.res_off : kBufOutside,
                                                            so + static_cast<uint32_t>((ni * 32 + q4 * 8) * 2), 0));
            }
    };
    if (has_res) res_load(0, rres[0]);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        if (RES_BUF == 2 && has_res && mi + 1 < MI) res_load(mi + 1, rres[(mi + 1) % RES_BUF]);
#pragma unroll
        for (int nc = 0; nc < NI / EPI_NI; ++nc) {
#pragma unroll
            for (int nh = 0; nh < EPI_NI; ++nh) {
                const int ni = nc * EPI_NI + nh;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 mul, add;
                    if constexpr (HOIST) {
                        mul = mulv[ni][q4];
                        add = addv[ni][q4];
                    } else {
                        mul = *reinterpret_cast<const f32x4*>(cmul + ni * 32 + q4 * 8 + lh * 4);
                        add = *reinterpret_cast<const f32x4*>(cadd + ni * 32 + q4 * 8 + lh * 4);
                    }
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[mi][ni][q4 * 4 + e] * mul[e] + add[e];
                    if (has_res) {
                        const u32x2 r2 = rres[mi % RES_BUF][ni][q4];
                        v[0] += __uint_as_float(r2[0] << 16);
                        v[1] += __uint_as_float(r2[0] & 0xFFFF0000u);
                        v[2] += __uint_as_float(r2[1] << 16);
                        v[3] += __uint_as_float(r2[1] & 0xFFFF0000u);
                    }
                    u32x2 pk;
                    pk[0] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(
                                                             __builtin_bit_cast(s16x2, pack_bf16x2(v[0], v[1])), floor2));
                    pk[1] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(
                                                             __builtin_bit_cast(s16x2, pack_bf16x2(v[2], v[3])), floor2));
                    *reinterpret_cast<u32x2*>(stg + lrow * EPI_ROW + (nh * 32 + q4 * 8 + lh * 4) * 2) = pk;
                }
            }
            if (RES_BUF == 1 && nc + 1 == NI / EPI_NI && has_res && mi + 1 < MI) res_load(mi + 1, rres[0]);
            // the same wave wrote and reads: LDS executes a wave's operations in order
            const uint32_t so = tile_off + static_cast<uint32_t>(mi * 32) * ldyB + static_cast<uint32_t>(nc * EPI_CH * 2);
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int row = it * RPI + lane / LPR;
                const int c16 = lane % LPR;
                const u32x4 val = *reinterpret_cast<const u32x4*>(stg + row * EPI_ROW + c16 * 16);
                const bool ok = FULL || (mi * 32 + row < rows_in && nc * EPI_CH + c16 * 8 < cols_in);
                // The tile offset is added to the lane offset instead of travelling in the scalar-offset field: for a
                // store of more than 8 bytes with a scalar offset the compiler adds no wait state before an
                // instruction that overwrites the data registers, and on this part such an overwrite in the very
                // next instruction was seen to reach memory in place of the first data dword.
                __builtin_amdgcn_raw_buffer_store_b128(val, ry, ok ? L.st_off[it] + so : kBufOutside, 0, kStoreThrough);
            }
        }
    }
}

// Dispatch on whether the wave's tile lies inside the tensor (wave-uniform).
template <int MI, int NI, int EPI_CH>
__device__ __forceinline__ void store_tile_bf16(const f32x16 (&acc)[MI][NI], const float* cmul, const float* cadd,
                                                unsigned char* stg, const TileStoreLane<EPI_CH>& L,
                                                __amdgpu_buffer_rsrc_t ry, __amdgpu_buffer_rsrc_t rr, bool has_res,
                                                uint32_t m_first, int n_first, uint32_t M, int NC, uint32_t ldyB,
                                                uint32_t relu_floor, int lane) {
    const bool full = m_first + MI * 32 <= M && n_first + NI * 32 <= NC;
    if (full)
        store_tile_bf16<MI, NI, EPI_CH, true>(acc, cmul, cadd, stg, L, ry, rr, has_res, m_first, n_first, M, NC, ldyB, relu_floor, lane);
    else
        store_tile_bf16<MI, NI, EPI_CH, false>(acc, cmul, cadd, stg, L, ry, rr, has_res, m_first, n_first, M, NC, ldyB, relu_floor, lane);
}

}  // namespace twn

