// Implicit-GEMM ternary convolution / inner product on gfx950 bf16 MFMA
// (Eq. 2, Alg. 1 step 8; the same kernel serves the backward-data pass of
// Alg. 1 step 9 through a re-expressed gather).
//
// Design, per workgroup tile BM (pixels) x BN (output channels), K slabs of 64:
//   * activations: 16-byte global loads (8 bf16 of one tap) -> LDS, rows of
//     128 bytes with the 16-byte chunk index XOR-swizzled by ((row >> 1) & 7), read
//     back with ds_read_b128 as the A operand of v_mfma_f32_32x32x16_bf16;
//   * weights never touch LDS: each lane loads the 32 packed codes (8 bytes)
//     of its own output channel and its own half of the K slab straight from
//     global memory (the packed bank is small and L2-resident) and expands
//     them in registers.  The twn2 format keeps even-k codes in the low
//     half-word and odd-k codes in the high half-word of each 32-bit word, and
//     a 2-bit field (non-zero, negative) shifted to bits [14,15] of a bf16 is
//     exactly {0, +2.0, -2.0}; so one shift and one AND produce two B-operand
//     elements.  The factor 2 is folded into alpha in the fp32 epilogue.
//   * MFMA k-slot mapping: in MFMA step kk (0..3) of a slab, lane-half h
//     (lane/32) carries k = 32h + 8kk .. +7 for both operands.
#include "twn_kernels.h"

namespace twn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

enum { kModeGemm = 0, kModeVec8 = 1, kModeScalar = 2 };

// Weight operand formats.  kFmtPacked is the product path; the other two exist to be measured against it:
// kFmtAlpha builds the paper's operand alpha*W~ itself (bf16 {-alpha, 0, +alpha}, alpha rounded to bf16)
// at expansion time instead of scaling the fp32 sum, kFmtInt8 reads weights stored one int8 per weight,
// kFmtSign1 reads the 1-bit sign codes of the binary-weight comparison (Sec. 3) and expands them to +-1.
enum { kFmtPacked = 0, kFmtAlpha = 1, kFmtInt8 = 2, kFmtSign1 = 3 };

template <int BM, int BN, int WM, int WN, int MODE, int BFMT>
__global__ __launch_bounds__(64 * WM * WN) void gather_gemm_mfma_kernel(const GatherGemm g) {
    constexpr int T = 64 * WM * WN;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int NLOAD = BM * 8 / T;
    constexpr int ROWSTEP = T / 8;
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "tile/wave mismatch");
    static_assert((BM * 8) % T == 0, "A tile must split evenly over threads");

    __shared__ __attribute__((aligned(16))) uint16_t lds[2][BM * 64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lh = lane >> 5;

    const int tiles_n = (g.NC + BN - 1) / BN;
    const int64_t tile_m = blockIdx.x / tiles_n;
    const int tile_n = static_cast<int>(blockIdx.x % tiles_n);
    const int64_t m0 = tile_m * BM;
    const int n0 = tile_n * BN;

    const uint16_t* __restrict__ X = static_cast<const uint16_t*>(g.X);
    const uint32_t* __restrict__ Wq = static_cast<const uint32_t*>(g.Wq);

    // ---- per-thread A-load slots: NLOAD rows, one 16-byte chunk (8 k) each ----
    const int kc = tid & 7;
    int64_t pixbase[NLOAD];
    int ih0[NLOAD], iw0[NLOAD];
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int row = (tid >> 3) + i * ROWSTEP;
        const int64_t m = m0 + row;
        if (m < g.M) {
            if (MODE == kModeGemm) {
                pixbase[i] = m;
                ih0[i] = 0;
                iw0[i] = 0;
            } else {
                const int ow = static_cast<int>(m % g.OW);
                const int64_t t = m / g.OW;
                const int oh = static_cast<int>(t % g.OH);
                const int64_t n = t / g.OH;
                pixbase[i] = n * g.IH * g.IW;
                ih0[i] = oh * g.sh - g.ph;
                iw0[i] = ow * g.sw - g.pw;
            }
        } else {
            pixbase[i] = 0;
            ih0[i] = -(1 << 28);   // fails every bounds test below
            iw0[i] = -(1 << 28);
        }
    }

    u32x4 areg[NLOAD];
    constexpr int BW = (BFMT == kFmtInt8) ? 4 : 1;   // 8-byte words of weights per lane, row and slab
    u32x2 breg[NI][BW], breg_next[NI][BW];

    auto tap_coord = [&](int base, int tap, int step, int div, int limit, int& out) -> bool {
        int t = base + tap * step;
        if (div > 1) {
            if (t < 0 || (t % div) != 0) return false;
            t /= div;
        }
        out = t;
        return static_cast<unsigned>(t) < static_cast<unsigned>(limit);
    };

    auto load_a = [&](int kt) {
        const int k = kt * 64 + kc * 8;
        if (MODE == kModeGemm) {
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) {
                const bool ok = (ih0[i] == 0) && (k < g.K);
                areg[i] = ok ? *reinterpret_cast<const u32x4*>(X + pixbase[i] * g.xs + k) : u32x4{0, 0, 0, 0};
            }
        } else if (MODE == kModeVec8) {
            const int rs = k / g.IC;
            const int c = k - rs * g.IC;
            const int r = rs / g.S;
            const int s = rs - r * g.S;
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) {
                int th, tw;
                bool ok = tap_coord(ih0[i], r, g.dh, g.divh, g.IH, th);
                ok = tap_coord(iw0[i], s, g.dw, g.divw, g.IW, tw) && ok;
                ok = ok && (k < g.K);
                areg[i] = ok ? *reinterpret_cast<const u32x4*>(
                                   X + (pixbase[i] + static_cast<int64_t>(th) * g.IW + tw) * g.xs + c)
                             : u32x4{0, 0, 0, 0};
            }
        } else if (g.plain_gemm) {
            // rows of X with a length that is not a multiple of 8: element loads, no tap arithmetic
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) {
                uint32_t w4[4] = {0, 0, 0, 0};
                const int64_t m = m0 + (tid >> 3) + i * ROWSTEP;      // GEMM row = pixel index
                const uint16_t* src = X + m * g.xs + k;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t v = (m < g.M && k + e < g.K) ? src[e] : 0u;
                    w4[e >> 1] |= v << ((e & 1) * 16);
                }
                areg[i] = u32x4{w4[0], w4[1], w4[2], w4[3]};
            }
        } else {
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) {
                uint32_t w4[4] = {0, 0, 0, 0};
                for (int e = 0; e < 8; ++e) {
                    const int ke = k + e;
                    uint32_t v = 0;
                    if (ke < g.K) {
                        const int rs = ke / g.IC;
                        const int c = ke - rs * g.IC;
                        const int r = rs / g.S;
                        const int s = rs - r * g.S;
                        int th, tw;
                        bool ok = tap_coord(ih0[i], r, g.dh, g.divh, g.IH, th);
                        ok = tap_coord(iw0[i], s, g.dw, g.divw, g.IW, tw) && ok;
                        if (ok) v = X[(pixbase[i] + static_cast<int64_t>(th) * g.IW + tw) * g.xs + c];
                    }
                    w4[e >> 1] |= v << ((e & 1) * 16);
                }
                areg[i] = u32x4{w4[0], w4[1], w4[2], w4[3]};
            }
        }
    };

    auto store_a = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            const int row = (tid >> 3) + i * ROWSTEP;
            const int chunk = kc ^ ((row >> 1) & 7);
            *reinterpret_cast<u32x4*>(&lds[buf][row * 64 + chunk * 8]) = areg[i];
        }
    };

    auto load_b = [&](int kt, u32x2 (*dst)[BW]) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int ncol = n0 + wn * TN + ni * 32 + lrow;
            if (BFMT == kFmtInt8) {
                // int8 [NC][K], K % 8 == 0: this lane's 8 weights of each of the four MFMA steps
                const uint8_t* wrow = reinterpret_cast<const uint8_t*>(g.Wq) + static_cast<int64_t>(ncol) * g.K;
#pragma unroll
                for (int kk = 0; kk < BW; ++kk) {
                    const int k = kt * 64 + lh * 32 + kk * 8;   // the k range of this lane's A fragment at step kk
                    dst[ni][kk] = (ncol < g.NC && k < g.K) ? *reinterpret_cast<const u32x2*>(wrow + k) : u32x2{0, 0};
                }
            } else if (BFMT == kFmtSign1) {
                // two words per row and slab; this lane's half of the slab (k = lh*32 .. +31) is one of them
                dst[ni][0] = u32x2{(ncol < g.NC) ? Wq[static_cast<int64_t>(ncol) * g.wpr + kt * 2 + lh] : 0u, 0u};
            } else {
                dst[ni][0] = (ncol < g.NC)
                                 ? *reinterpret_cast<const u32x2*>(Wq + static_cast<int64_t>(ncol) * g.wpr + kt * 4 + 2 * lh)
                                 : u32x2{0, 0};
            }
        }
    };

    // kFmtAlpha: bf16(alpha) of this lane's output channels, in both halves of a register
    uint32_t alpha2[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int ncol = n0 + wn * TN + ni * 32 + lrow;
        const uint32_t ab = (BFMT == kFmtAlpha && ncol < g.NC) ? f32_to_bf16(g.alpha[ncol / g.rows_per_group]) : 0u;
        alpha2[ni] = ab | (ab << 16);
    }

    // the 8 weights of (channel tile ni, MFMA step kk) as four registers of two bf16 each
    auto expand = [&](int ni, int kk) -> u32x4 {
        u32x4 b;
        if (BFMT == kFmtInt8) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                // bytes 0x01 / 0xFF / 0x00 -> 0x40 / 0xC0 / 0x00, the high byte of bf16 +2 / -2 / 0
                const uint32_t x = breg[ni][kk][h];
                const uint32_t y = ((x << 6) & 0x40404040u) | (x & 0x80808080u);
                b[2 * h] = __builtin_amdgcn_perm(0u, y, 0x010C000Cu);       // [0, y.b0, 0, y.b1]
                b[2 * h + 1] = __builtin_amdgcn_perm(0u, y, 0x030C020Cu);   // [0, y.b2, 0, y.b3]
            }
        } else if (BFMT == kFmtSign1) {
            // weights k = 8*kk + 2r (bit 4*kk + r) and 8*kk + 2r + 1 (bit 16 + 4*kk + r): sign bits onto bf16 1.0
            const uint32_t word = breg[ni][0][0];
#pragma unroll
            for (int r = 0; r < 4; ++r) b[r] = ((word << (15 - (kk * 4 + r))) & 0x80008000u) | 0x3F803F80u;
        } else {
            const uint32_t word = breg[ni][0][kk >> 1];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = (kk & 1) * 4 + r;
                if (BFMT == kFmtAlpha) {
                    // sign from bit 1 of the field; bit 0 (nonzero) widened to a 16-bit mask that gates alpha
                    const uint32_t sign = (word << (14 - 2 * i)) & 0x80008000u;
                    const s16x2 nz = __builtin_bit_cast(s16x2, word << (15 - 2 * i)) >> 15;
                    b[r] = (__builtin_bit_cast(uint32_t, nz) & alpha2[ni]) | sign;
                } else {
                    b[r] = (word << (14 - 2 * i)) & 0xC000C000u;
                }
            }
        }
        return b;
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.0f;

    const int KT = (g.K + 63) / 64;
    load_a(0);
    load_b(0, breg_next);
    store_a(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int w = 0; w < BW; ++w) breg[ni][w] = breg_next[ni][w];
        const bool more = (kt + 1 < KT);
        if (more) {
            load_a(kt + 1);
            load_b(kt + 1, breg_next);
        }
        // A fragments are fetched one MFMA step ahead of their use
        bf16x8 afrag[2][MI];
        auto read_a = [&](int kk, bf16x8* dst) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int row = wm * TM + mi * 32 + lrow;
                const int chunk = (lh * 4 + kk) ^ ((row >> 1) & 7);
                dst[mi] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(&lds[cur][row * 64 + chunk * 8]));
            }
        };
        read_a(0, afrag[0]);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk + 1 < 4) read_a(kk + 1, afrag[(kk + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads ahead of this step's MFMAs
            bf16x8 bfrag[NI];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) bfrag[ni] = __builtin_bit_cast(bf16x8, expand(ni, kk));
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[kk & 1][mi], bfrag[ni], acc[mi][ni], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more) store_a(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: y = relu?((alpha*acc)*scale + shift + residual) ----
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int ncol = n0 + wn * TN + ni * 32 + lrow;
        if (ncol >= g.NC) continue;
        // codes were expanded to +-2 (or, for kFmtAlpha, to +-alpha already)
        const float al = (BFMT == kFmtAlpha) ? 1.0f : (BFMT == kFmtSign1 ? 1.0f : 0.5f) * g.alpha[ncol / g.rows_per_group];
        const float sc = g.scale ? g.scale[ncol] : 1.0f;
        const float sf = g.shift ? g.shift[ncol] : 0.0f;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t m = m0 + wm * TM + mi * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
                if (m >= g.M) continue;
                float v = (acc[mi][ni][e] * al) * sc + sf;
                const int64_t off = m * g.ldy + ncol;
                if (g.y_f32) {
                    if (g.residual) v += static_cast<const float*>(g.residual)[off];
                    if (g.relu) v = fmaxf(v, 0.0f);
                    static_cast<float*>(g.Y)[off] = v;
                } else {
                    if (g.residual) v += bf16_to_f32(static_cast<const uint16_t*>(g.residual)[off]);
                    if (g.relu) v = fmaxf(v, 0.0f);
                    static_cast<uint16_t*>(g.Y)[off] = f32_to_bf16(v);
                }
            }
        }
    }
}

__device__ __forceinline__ void pad_c4_body(const uint16_t* __restrict__ X, int N, int H, int W, int C, int ph, int pw,
                                            int Hp, int Wp, uint16_t* __restrict__ Xp, int64_t block) {
    const int64_t id = block * blockDim.x + threadIdx.x;
    const int64_t total = static_cast<int64_t>(N) * Hp * Wp;
    if (id >= total) return;
    const int wp = static_cast<int>(id % Wp);
    const int64_t t = id / Wp;
    const int hp = static_cast<int>(t % Hp);
    const int64_t n = t / Hp;
    const int h = hp - ph, w = wp - pw;
    uint32_t v[4] = {0, 0, 0, 0};
    if (static_cast<unsigned>(h) < static_cast<unsigned>(H) && static_cast<unsigned>(w) < static_cast<unsigned>(W)) {
        const uint16_t* src = X + ((n * H + h) * W + w) * C;
        for (int c = 0; c < C; ++c) v[c] = src[c];
    }
    u32x2 o;
    o[0] = v[0] | (v[1] << 16);
    o[1] = v[2] | (v[3] << 16);
    *reinterpret_cast<u32x2*>(Xp + id * 4) = o;
}

__global__ __launch_bounds__(256) void pad_c4_kernel(const uint16_t* __restrict__ X, int N, int H, int W, int C,
                                                     int ph, int pw, int Hp, int Wp, uint16_t* __restrict__ Xp) {
    pad_c4_body(X, N, H, W, C, ph, pw, Hp, Wp, Xp, blockIdx.x);
}

__device__ __forceinline__ void repack_c4_body(const uint32_t* __restrict__ packed, int rows, int C, int R, int S, int Sp,
                                               int wpr, int wpr2, uint32_t* __restrict__ out, int64_t block) {
    const int64_t id = block * blockDim.x + threadIdx.x;
    if (id >= static_cast<int64_t>(rows) * wpr2) return;
    const int row = static_cast<int>(id / wpr2), j = static_cast<int>(id % wpr2);
    uint32_t word = 0;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int k2 = j * 16 + t;
        const int c = k2 & 3, rs = k2 >> 2;
        const int s = rs % Sp, r = rs / Sp;
        if (c < C && s < S && r < R) {
            const int k = (r * S + s) * C + c;
            const uint32_t src = packed[static_cast<int64_t>(row) * wpr + (k >> 4)];
            const int tt = k & 15;
            const uint32_t fld = (src >> ((tt & 1) * 16 + (tt >> 1) * 2)) & 3u;
            word |= fld << ((t & 1) * 16 + (t >> 1) * 2);
        }
    }
    out[id] = word;
}

// Both preparations of the first-layer path in one launch: the first pad_blocks workgroups copy X, the rest
// re-order the codes (the two are independent, and a launch costs more than either of them).
__global__ __launch_bounds__(256) void pad_repack_c4_kernel(const uint16_t* __restrict__ X, int N, int H, int W, int C,
                                                            int ph, int pw, int Hp, int Wp, uint16_t* __restrict__ Xp,
                                                            unsigned pad_blocks, const uint32_t* __restrict__ packed,
                                                            int rows, int R, int S, int Sp, int wpr, int wpr2,
                                                            uint32_t* __restrict__ out) {
    if (blockIdx.x < pad_blocks)
        pad_c4_body(X, N, H, W, C, ph, pw, Hp, Wp, Xp, blockIdx.x);
    else
        repack_c4_body(packed, rows, C, R, S, Sp, wpr, wpr2, out, blockIdx.x - pad_blocks);
}

int32_t launch_pad_repack_c4(const uint16_t* X, int N, int H, int W, int C, int ph, int pw, int Hp, int Wp, uint16_t* Xp,
                             const uint32_t* packed, int rows, int R, int S, int Sp, uint32_t* out, hipStream_t st) {
    const int64_t total_x = static_cast<int64_t>(N) * Hp * Wp;
    const int wpr = static_cast<int>(twn_packed_words_per_row(static_cast<int64_t>(R) * S * C));
    const int wpr2 = static_cast<int>(twn_packed_words_per_row(static_cast<int64_t>(R) * Sp * 4));
    const int64_t total_w = static_cast<int64_t>(rows) * wpr2;
    const int64_t pad_blocks = (total_x + 255) / 256, blocks = pad_blocks + (total_w + 255) / 256;
    if (blocks >= (1LL << 31)) return TWN_ERR_SHAPE;
    pad_repack_c4_kernel<<<static_cast<unsigned>(blocks), 256, 0, st>>>(X, N, H, W, C, ph, pw, Hp, Wp, Xp,
                                                                     static_cast<unsigned>(pad_blocks), packed, rows, R, S,
                                                                     Sp, wpr, wpr2, out);
    return launch_status();
}

// Backward-data with one alpha per group of filters (Alg. 1 steps 3-7 feeding step 9): alpha multiplies per forward
// output channel o, which is a reduction index of dX, so it cannot be applied after the sum.  dY is scaled instead.
// The product v = dY[p][o] * alpha[o / rows_per_group] (float32) is carried as two bf16 terms, hi = bf16(v) and
// lo = bf16(v - hi), which together hold v to about 2^-17: the contraction runs once over each (alpha = 1, which
// thread 0 writes to `one`), the second pass adding onto the first, and no rounding of the inputs is added.
__global__ __launch_bounds__(256) void scale_channels_kernel(const uint16_t* __restrict__ dY, const float* __restrict__ alpha,
                                                             int rows_per_group, int O, int64_t total,
                                                             uint16_t* __restrict__ hi, uint16_t* __restrict__ lo,
                                                             float* __restrict__ one) {
    const int64_t id = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (id == 0) *one = 1.0f;
    if (id >= total) return;
    const int o = static_cast<int>(id % O);
    const float v = bf16_to_f32(dY[id]) * alpha[o / rows_per_group];
    const uint16_t h = f32_to_bf16(v);
    hi[id] = h;
    lo[id] = f32_to_bf16(v - bf16_to_f32(h));
}

int32_t launch_scale_channels(const uint16_t* dY, const float* alpha, int rows_per_group, int O, int64_t pixels,
                              uint16_t* hi, uint16_t* lo, float* one, hipStream_t st) {
    const int64_t total = pixels * O;
    if (total <= 0 || (total + 255) / 256 >= (1LL << 31)) return TWN_ERR_SHAPE;
    scale_channels_kernel<<<static_cast<unsigned>((total + 255) / 256), 256, 0, st>>>(dY, alpha, rows_per_group, O, total,
                                                                                   hi, lo, one);
    return launch_status();
}

// Strided backward-data as one stride-1 problem per residue class of the output pixels: the taps that reach
// class (a, b) are r = r0 + jr*sh, s = s0 + js*sw.  Their codes are gathered from the transposed copy into a
// contiguous K range per class: out[class][c][(jr*ns + js)*O/16 + t] = packed_T[c][((r0+jr*sh)*S + s0+js*sw)*O/16 + t].
__global__ __launch_bounds__(256) void gather_class_codes_kernel(const uint32_t* __restrict__ packed_T, int C, int wprT, int S,
                                                                 int O16, int sh, int sw, DxClassTable tb,
                                                                 uint32_t* __restrict__ out) {
    const int64_t id = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    int k = 0;
    while (k + 1 < tb.count && id >= tb.first_word[k + 1]) ++k;
    const int64_t local = id - tb.first_word[k];
    const int wpr = tb.wpr[k];
    if (k >= tb.count || local >= static_cast<int64_t>(C) * wpr) return;
    const int c = static_cast<int>(local / wpr), j = static_cast<int>(local % wpr);
    uint32_t word = 0u;
    if (j < tb.nr[k] * tb.ns[k] * O16) {
        const int tap = j / O16, t = j % O16;
        const int jr = tap / tb.ns[k], js = tap % tb.ns[k];
        const int src_tap = (tb.r0[k] + jr * sh) * S + tb.s0[k] + js * sw;
        word = packed_T[static_cast<int64_t>(c) * wprT + static_cast<int64_t>(src_tap) * O16 + t];
    }
    out[id] = word;
}

int32_t launch_gather_class_codes(const uint32_t* packed_T, int C, int wprT, int S, int O, int sh, int sw,
                                  const DxClassTable& tb, int64_t total_words, uint32_t* out, hipStream_t st) {
    if (total_words <= 0 || (total_words + 255) / 256 >= (1LL << 31)) return TWN_ERR_SHAPE;
    gather_class_codes_kernel<<<static_cast<unsigned>((total_words + 255) / 256), 256, 0, st>>>(packed_T, C, wprT, S, O / 16,
                                                                                             sh, sw, tb, out);
    return launch_status();
}

// Zero fill in 16-byte units (a kernel rather than a memset, so that callers may capture it into a graph).
__global__ __launch_bounds__(256) void zero_fill_kernel(u32x4* __restrict__ p, int64_t n16) {
    const int64_t id = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (id < n16) p[id] = u32x4{0u, 0u, 0u, 0u};
}

int32_t launch_zero_fill(void* p, int64_t bytes, hipStream_t st) {
    const int64_t n16 = bytes / 16;
    if (bytes % 16 != 0 || n16 <= 0 || (n16 + 255) / 256 >= (1LL << 31)) return TWN_ERR_SHAPE;
    zero_fill_kernel<<<static_cast<unsigned>((n16 + 255) / 256), 256, 0, st>>>(static_cast<u32x4*>(p), n16);
    return launch_status();
}

int32_t launch_pad_c4(const uint16_t* X, int N, int H, int W, int C, int ph, int pw, int Hp, int Wp,
                      uint16_t* Xp, hipStream_t st) {
    const int64_t total = static_cast<int64_t>(N) * Hp * Wp;
    if (total <= 0 || (total + 255) / 256 >= (1LL << 31)) return TWN_ERR_SHAPE;
    pad_c4_kernel<<<static_cast<unsigned>((total + 255) / 256), 256, 0, st>>>(X, N, H, W, C, ph, pw, Hp, Wp, Xp);
    return launch_status();
}

template <int BM, int BN, int WM, int WN, int BFMT = kFmtPacked>
static int32_t launch_tile(const GatherGemm& g, int mode, hipStream_t st) {
    const int64_t tiles_m = (g.M + BM - 1) / BM;
    const int64_t tiles_n = (g.NC + BN - 1) / BN;
    const int64_t blocks = tiles_m * tiles_n;
    if (blocks <= 0 || blocks >= (1LL << 31)) return TWN_ERR_SHAPE;
    const dim3 grid(static_cast<unsigned>(blocks));
    const dim3 block(64 * WM * WN);
    switch (mode) {
        case kModeGemm: gather_gemm_mfma_kernel<BM, BN, WM, WN, kModeGemm, BFMT><<<grid, block, 0, st>>>(g); break;
        case kModeVec8: gather_gemm_mfma_kernel<BM, BN, WM, WN, kModeVec8, BFMT><<<grid, block, 0, st>>>(g); break;
        default: gather_gemm_mfma_kernel<BM, BN, WM, WN, kModeScalar, BFMT><<<grid, block, 0, st>>>(g); break;
    }
    return launch_status();
}

static int gather_mode(const GatherGemm& g) {
    if (g.chunk_gather) return kModeVec8;
    if (g.IC % 8 != 0 || g.xs % 8 != 0) return kModeScalar;
    return g.plain_gemm ? kModeGemm : kModeVec8;
}

int32_t gather_gemm_splits(const GatherGemm& g) {
    // split K when even 64x128 tiles leave half the CUs idle and K is deep enough to share out (few workgroups
    // with two slabs in flight each are bound by memory latency when their input is not in L2)
    if (gather_mode(g) == kModeScalar || env_int("TWN_TILE", 0) != 0) return 1;
    const int64_t blocks = ((g.M + 127) / 128) * ((g.NC + 127) / 128);
    const int64_t blocks64 = ((g.M + 63) / 64) * ((g.NC + 127) / 128);
    const int KT = (g.K + 63) / 64;
    // below 16 slabs the persistent kernel with K groups inside the workgroup does it in one launch
    // (ResNet-18 classifier, 64 x 1000 x 512: 11 us in two launches -> 5 us)
    if (blocks64 >= 128 || KT < 16) return 1;
    int64_t splits = (448 + blocks - 1) / blocks;
    if (splits > KT / 4) splits = KT / 4;
    if (splits > 32) splits = 32;
    if (splits < 1) splits = 1;
    // every range must own at least one slab
    const int kps = static_cast<int>((KT + splits - 1) / splits);
    return static_cast<int32_t>((KT + kps - 1) / kps);
}

// Tile id launch_gather_gemm_mfma would give an unsplit problem in the one-tile-per-workgroup direct-to-LDS kernel,
// or 0 when the problem would not run there (scalar gathers, forced tiles; persistent kernels unless
// `instead_of_persistent` asks for the tile the problem would get if they did not exist).
int32_t gather_gemm_dma_tile(const GatherGemm& g, bool instead_of_persistent) {
    if (gather_mode(g) == kModeScalar || env_int("TWN_TILE", 0) != 0 || g.splits > 1) return 0;
    if (!instead_of_persistent && env_int("TWN_STREAM", 1) != 0 && conv_stream_applicable(g)) return 0;
    auto blocks = [&](int bm, int bn) { return ((g.M + bm - 1) / bm) * ((g.NC + bn - 1) / bn); };
    int tile;
    if (g.NC <= 64) tile = 16;
    else if (g.NC <= 128) tile = 12;
    else tile = (blocks(128, 256) >= 512) ? 17 : 12;
    if (tile == 12 && blocks(128, 128) <= 256) tile = 14;
    if (tile == 12) tile = 15;
    return tile;
}

int32_t launch_gather_gemm_mfma(const GatherGemm& g, int variant, hipStream_t st) {
    const int mode = gather_mode(g);
    // the comparison variants run in the register-staged 128x128 kernel only
    if (variant == TWN_VAR_BF16_ALPHA_LDS) return launch_tile<128, 128, 2, 2, kFmtAlpha>(g, mode, st);
    if (variant == TWN_VAR_I8_STORED_POSTSCALE) {
        if (g.K % 8 != 0) return TWN_ERR_UNSUPPORTED;
        return launch_tile<128, 128, 2, 2, kFmtInt8>(g, mode, st);
    }
    if (variant == TWN_VAR_BF16_SIGN1_POSTSCALE) return launch_tile<128, 128, 2, 2, kFmtSign1>(g, mode, st);
    if (variant != TWN_VAR_BF16_POSTSCALE) return TWN_ERR_UNSUPPORTED;

    // Tile choice: the largest tile that still gives every CU work; narrow N tiles for narrow layers.
    int tile = env_int("TWN_TILE", 0);
    // 3x3 stride-1 layers over 64 channels: weights resident in registers, input patches with halo in LDS
    if (tile == 0 && env_int("TWN_C64", 1) != 0 && conv_c64_applicable(g)) return launch_conv_c64(g, st);
    if (mode != kModeScalar && (tile == 0 || tile > 10)) {
        // multi-stage direct-to-LDS kernel
        if (tile == 0) {
            auto blocks = [&](int bm, int bn) { return ((g.M + bm - 1) / bm) * ((g.NC + bn - 1) / bn); };
            if (g.splits > 1) tile = 12;
            else if (g.NC <= 64) tile = 16;
            else if (g.NC <= 128) tile = 12;
            else tile = (blocks(128, 256) >= 512) ? 17 : 12;
            // at most one 128x128 workgroup per CU: 64x128 tiles double the workgroups (layers with few pixels)
            if (tile == 12 && g.splits == 1 && blocks(128, 128) <= 256) tile = 14;
            // unsplit 128x128 tiles: waves side by side (128x32 each) expand every code once per workgroup
            // instead of twice; a few percent faster than the 2x2 arrangement, which keeps the split-K builds
            if (tile == 12 && g.splits == 1) tile = 15;
        }
        if ((tile == 12 || (tile >= 14 && tile <= 17)) && env_int("TWN_STREAM", 1) != 0 && conv_stream_applicable(g))
            return launch_conv_stream(g, tile, st);
        return launch_gather_gemm_dma(g, tile, st);
    }
    if (tile > 10) tile = 0;   // ids above 10 name tiles of the direct-to-LDS kernel
    if (tile == 0) {
        auto blocks = [&](int bm, int bn) { return ((g.M + bm - 1) / bm) * ((g.NC + bn - 1) / bn); };
        const int64_t want = 256;
        if (g.NC <= 64) tile = (blocks(256, 64) >= want) ? 3 : 5;
        else if (g.NC <= 128) tile = (blocks(256, 128) >= want) ? 2 : 4;
        else if (blocks(256, 256) >= want) tile = 1;
        else if (blocks(256, 128) >= want) tile = 2;
        else tile = 4;
    }
    switch (tile) {
        case 1: return launch_tile<256, 256, 2, 2>(g, mode, st);
        case 2: return launch_tile<256, 128, 2, 2>(g, mode, st);
        case 3: return launch_tile<256, 64, 4, 1>(g, mode, st);
        case 4: return launch_tile<128, 128, 2, 2>(g, mode, st);
        case 5: return launch_tile<128, 64, 4, 1>(g, mode, st);
        case 6: return launch_tile<256, 256, 2, 4>(g, mode, st);
        default: return TWN_ERR_UNSUPPORTED;
    }
}

}  // namespace twn
