// Multiplication-free ternary convolution / inner product on the vector ALUs, gfx950 (Eq. 2: the operation the
// paper writes as (alpha X) (+) W^t; Sec. 2.1 "Computational requirement": a ternary weight needs no multiply and a
// zero weight no work at all).  Comparison variant TWN_VAR_ADDSUB_SPARSE: the measured counterpart of the
// matrix-core kernels, which spend a dense multiply-accumulate on every code, zero or not.
//
// Mapping.  The codes of a filter are the same for every pixel, so with pixels across the lanes of a wave the
// sparsity pattern is wave-uniform: a wave walks the non-zero codes of one filter row with scalar instructions
// (find-first-set over the +1 mask and over the -1 mask of each packed word, derived from the 2-bit fields with
// three scalar bit operations) and issues, per non-zero code, ONE 16-byte LDS read (the activations of its four
// pixels per lane at that k) and FOUR float32 additions or subtractions.  Zero codes cost nothing and no branch
// diverges.  The accumulators are float32; the only multiplications are those of the epilogue (alpha and the
// block tail, once per output).
//
// A workgroup of 16 waves owns 256 pixels x 64 filters (32 or 16 for layers with few pixels).  Per 64-wide K slab it stages the activations, widened to
// float32 and transposed to [k][pixel], in 64 KB of LDS (lanes of a wave write consecutive pixels of one k: no
// bank conflicts), then every wave accumulates its filters (4, 2 or 1) over the slab.  Two workgroups share a CU (32
// waves): while one stages, the other adds, and 8 waves per SIMD cover the read-to-add latency of the walk.
// Packed codes are the library's ordinary 2-bit format; there is no index structure to build.
#include "twn_kernels.h"
#include "twn_mfma.h"

namespace twn {

namespace {
constexpr int kAsBM = 256;                    // pixels per workgroup (4 per lane)
constexpr int kAsWaves = 16;
constexpr int kAsLds = 64 * kAsBM * 4;        // one K slab of float32 activations
}  // namespace

// kAsCh filters per wave: a workgroup owns 256 pixels x 16 * kAsCh filters
template <int kAsCh>
__global__ __launch_bounds__(64 * kAsWaves, 8) void conv_addsub_kernel(const GatherGemm g) {
    constexpr int kAsBN = kAsWaves * kAsCh;
    extern __shared__ __attribute__((aligned(16))) float xs[];      // [64 k][256 pixels]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_n = (g.NC + kAsBN - 1) / kAsBN;
    const int64_t m0 = static_cast<int64_t>(blockIdx.x / tiles_n) * kAsBM;
    const int n0 = static_cast<int>(blockIdx.x % tiles_n) * kAsBN;
    const uint16_t* __restrict__ X = static_cast<const uint16_t*>(g.X);
    const uint32_t* __restrict__ Wq = static_cast<const uint32_t*>(g.Wq);

    // staging role: pixel p of the tile, chunks 2*cg and 2*cg+1 (8 channels each) of every slab
    const int p = tid & (kAsBM - 1);
    const int cg = tid >> 8;
    const int64_t am = m0 + p;
    int64_t pixbase = 0;
    int ih0 = -(1 << 28), iw0 = -(1 << 28);
    if (am < g.M) {
        const int ow = static_cast<int>(am % g.OW);
        const int64_t t = am / g.OW;
        const int oh = static_cast<int>(t % g.OH);
        pixbase = (t / g.OH) * g.IH * g.IW;
        ih0 = oh * g.sh - g.ph;
        iw0 = ow * g.sw - g.pw;
    }
    const int cpt = g.IC / 8;                  // 8-channel chunks per filter tap

    f32x4 acc[kAsCh];
#pragma unroll
    for (int j = 0; j < kAsCh; ++j) acc[j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int KT = (g.K + 63) / 64;
    for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int ch = cg * 2 + h;
            const int q = kt * 8 + ch;          // chunk of K
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (q * 8 < g.K) {
                const int tap = q / cpt;
                const int c0 = (q - tap * cpt) * 8;
                const int r = tap / g.S;
                const int s = tap - r * g.S;
                const int th = ih0 + r * g.dh, tw = iw0 + s * g.dw;
                if (static_cast<unsigned>(th) < static_cast<unsigned>(g.IH) &&
                    static_cast<unsigned>(tw) < static_cast<unsigned>(g.IW))
                    raw = *reinterpret_cast<const u32x4*>(X + (pixbase + static_cast<int64_t>(th) * g.IW + tw) * g.xs + c0);
            }
            float* dst = xs + (ch * 8) * kAsBM + p;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dst[(2 * e) * kAsBM] = __uint_as_float(raw[e] << 16);            // bf16 -> float32 is a shift
                dst[(2 * e + 1) * kAsBM] = __uint_as_float(raw[e] & 0xFFFF0000u);
            }
        }
        __syncthreads();

        const f32x4* xv = reinterpret_cast<const f32x4*>(xs) + lane;           // pixels 4*lane .. 4*lane+3 of row k: xv[k * 64]
#pragma unroll
        for (int j = 0; j < kAsCh; ++j) {
            const int n = n0 + wave * kAsCh + j;
            u32x4 cw = {0u, 0u, 0u, 0u};
            if (n < g.NC) cw = *reinterpret_cast<const u32x4*>(Wq + static_cast<int64_t>(n) * g.wpr + kt * 4);
#pragma unroll
            for (int wp = 0; wp < 2; ++wp) {
                // Word j of the slab holds k = 16j+2i in bits [2i, 2i+1] and k = 16j+2i+1 in bits [16+2i, 17+2i].  The low
                // halves of words 2wp, 2wp+1 side by side are the codes of the even k of 32 weights with field position
                // = k - 32wp, the high halves those of the odd k with position = k - 32wp - 1: the walk needs no further
                // index arithmetic (the constant part of the address is the read's immediate offset).
                const uint32_t w0 = __builtin_amdgcn_readfirstlane(cw[2 * wp]);
                const uint32_t w1 = __builtin_amdgcn_readfirstlane(cw[2 * wp + 1]);
#pragma unroll
                for (int odd = 0; odd < 2; ++odd) {
                    const uint32_t m = odd ? ((w0 >> 16) | (w1 & 0xFFFF0000u)) : ((w0 & 0xFFFFu) | (w1 << 16));
                    const uint32_t nz = m & 0x55555555u;
                    const uint32_t neg = (m >> 1) & 0x55555555u;
                    uint32_t plus = nz & ~neg, minus = nz & neg;
                    const f32x4* xk = xv + (32 * wp + odd) * (kAsBM / 4);
                    while (plus) {
                        const int pos = __builtin_ctz(plus);
                        plus &= plus - 1;
                        acc[j] += xk[pos * (kAsBM / 4)];
                    }
                    while (minus) {
                        const int pos = __builtin_ctz(minus);
                        minus &= minus - 1;
                        acc[j] -= xk[pos * (kAsBM / 4)];
                    }
                }
            }
        }
        __syncthreads();
    }

    // epilogue: alpha and the block tail, once per output
#pragma unroll
    for (int j = 0; j < kAsCh; ++j) {
        const int n = n0 + wave * kAsCh + j;
        if (n >= g.NC) continue;
        const float al = g.alpha[n / g.rows_per_group];
        const float sc = g.scale ? g.scale[n] : 1.0f;
        const float sf = g.shift ? g.shift[n] : 0.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t m = m0 + lane * 4 + e;
            if (m >= g.M) continue;
            float v = (acc[j][e] * al) * sc + sf;
            const int64_t off = m * g.ldy + n;
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

bool conv_addsub_applicable(const GatherGemm& g) {
    if (g.divh != 1 || g.divw != 1 || g.orU != 0 || g.splits > 1 || g.chunk_gather) return false;
    if (g.IC % 8 != 0 || g.xs % 8 != 0 || g.K % 8 != 0) return false;
    return aligned(g.X, 16) && aligned(g.Wq, 16);
}

int32_t launch_conv_addsub(const GatherGemm& g, hipStream_t st) {
    if (!conv_addsub_applicable(g)) return TWN_ERR_UNSUPPORTED;
    // four filters per wave amortise the staging of a slab best; layers with few pixels take fewer filters per
    // workgroup so that the grid still gives every CU its two workgroups
    const int64_t tiles_m = (g.M + kAsBM - 1) / kAsBM;
    auto blocks = [&](int bn) { return tiles_m * ((g.NC + bn - 1) / bn); };
    const int ch = blocks(64) >= 400 ? 4 : (blocks(32) >= 400 ? 2 : 1);
    const int64_t nb = blocks(16 * ch);
    if (nb <= 0 || nb >= (1LL << 31)) return TWN_ERR_SHAPE;
    const dim3 grid(static_cast<unsigned>(nb)), block(64 * kAsWaves);
    switch (ch) {
        case 4: conv_addsub_kernel<4><<<grid, block, kAsLds, st>>>(g); break;
        case 2: conv_addsub_kernel<2><<<grid, block, kAsLds, st>>>(g); break;
        default: conv_addsub_kernel<1><<<grid, block, kAsLds, st>>>(g); break;
    }
    return launch_status();
}

}  // namespace twn
