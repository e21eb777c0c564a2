// float32 path of the ternary convolution / inner product (Eq. 2, Alg. 1 step 8)
// for float32 activations: LDS-tiled implicit GEMM on the vector ALUs.  Inputs
// and outputs are float32; the running sums are kept in float64 (products with
// a code are exact, so only the additions round) because float32 accumulation
// of cancelling sums cannot hold a 1e-5 relative bound on small outputs.
// Weights are the same packed twn2 codes, expanded to {-1, 0, +1} floats while
// staging the tile; alpha is applied afterwards.
// The layers that use it (LeNet-sized) are launch-bound, so the kernel is kept
// simple: 64x64 output tile, K slabs of 16, 4x4 outputs per thread.
#include "twn_kernels.h"

namespace twn {

constexpr int kF32Tile = 64;
constexpr int kF32K = 16;

__global__ __launch_bounds__(256) void gather_gemm_fp32_kernel(const GatherGemm g) {
    __shared__ float As[kF32K][kF32Tile + 4];
    __shared__ float Bs[kF32K][kF32Tile + 4];

    const int tid = threadIdx.x;
    const int tiles_n = (g.NC + kF32Tile - 1) / kF32Tile;
    const int64_t m0 = static_cast<int64_t>(blockIdx.x / tiles_n) * kF32Tile;
    const int n0 = static_cast<int>(blockIdx.x % tiles_n) * kF32Tile;
    const float* __restrict__ X = static_cast<const float*>(g.X);
    const uint32_t* __restrict__ Wq = static_cast<const uint32_t*>(g.Wq);

    // A staging: thread loads the 4 consecutive k of one row
    const int arow = tid >> 2;
    const int akq = (tid & 3) * 4;
    const int64_t am = m0 + arow;
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
    // B staging: thread expands 4 consecutive codes of one output channel
    const int bcol = tid >> 2;
    const int bn = n0 + bcol;

    const int ty = tid >> 4, tx = tid & 15;
    double acc[4][4] = {};

    for (int k0 = 0; k0 < g.K; k0 += kF32K) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = k0 + akq + e;
            float v = 0.0f;
            if (k < g.K) {
                const int rs = k / g.IC;
                const int c = k - rs * g.IC;
                const int r = rs / g.S;
                const int s = rs - r * g.S;
                int th = ih0 + r * g.dh, tw = iw0 + s * g.dw;
                bool ok = true;
                if (g.divh > 1) { ok = ok && th >= 0 && (th % g.divh) == 0; th /= g.divh; }
                if (g.divw > 1) { ok = ok && tw >= 0 && (tw % g.divw) == 0; tw /= g.divw; }
                ok = ok && static_cast<unsigned>(th) < static_cast<unsigned>(g.IH) &&
                     static_cast<unsigned>(tw) < static_cast<unsigned>(g.IW);
                if (ok) v = X[(pixbase + static_cast<int64_t>(th) * g.IW + tw) * g.xs + c];
            }
            As[akq + e][arow] = v;
        }
        {
            const int k = k0 + akq;   // multiple of 4: the 4 codes sit in one word
            uint32_t word = 0;
            if (bn < g.NC && k < g.K) word = Wq[static_cast<int64_t>(bn) * g.wpr + (k >> 4)];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int t = (k + e) & 15;
                const uint32_t fld = (word >> ((t & 1) * 16 + (t >> 1) * 2)) & 3u;
                Bs[akq + e][bcol] = (fld & 1u) ? ((fld & 2u) ? -1.0f : 1.0f) : 0.0f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kF32K; ++k) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = static_cast<double>(As[k][ty * 4 + i]);
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = static_cast<double>(Bs[k][tx * 4 + j]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int ncol = n0 + tx * 4 + j;
        if (ncol >= g.NC) continue;
        const float al = g.alpha[ncol / g.rows_per_group];
        const float sc = g.scale ? g.scale[ncol] : 1.0f;
        const float sf = g.shift ? g.shift[ncol] : 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t m = m0 + ty * 4 + i;
            if (m >= g.M) continue;
            float v = (static_cast<float>(acc[i][j]) * al) * sc + sf;
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

int32_t launch_gather_gemm_fp32(const GatherGemm& g, hipStream_t st) {
    const int64_t blocks = ((g.M + kF32Tile - 1) / kF32Tile) * ((g.NC + kF32Tile - 1) / kF32Tile);
    if (blocks <= 0 || blocks >= (1LL << 31)) return TWN_ERR_SHAPE;
    gather_gemm_fp32_kernel<<<static_cast<unsigned>(blocks), 256, 0, st>>>(g);
    return launch_status();
}

}  // namespace twn
