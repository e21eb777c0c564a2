// float32 path of the ternary convolution / inner product (Eq. 2, Alg. 1 step 8)
// for float32 activations: LDS-tiled implicit GEMM on the vector ALUs.  Inputs
// and outputs are float32; the running sums are kept in float64 (products with
// a code are exact, so only the additions round) because float32 accumulation
// of cancelling sums cannot hold a 1e-5 relative bound on small outputs.
// Weights are the same packed twn2 codes, expanded to {-1, 0, +1} floats while
// staging the tile; alpha is applied afterwards.
// The layers that use it (LeNet-sized) are small, so the kernel is kept simple, but two things matter even
// there: the gathers of the next K slab are in flight (in registers) while the current slab is multiplied, and
// problems with few 64x64 tiles (the fully-connected layers at batch 64) run 32x32 tiles, four times as many
// workgroups.  A thread owns (TS/16)^2 outputs.
#include "twn_kernels.h"

namespace twn {

template <int TS>
__global__ __launch_bounds__(256) void gather_gemm_fp32_kernel(const GatherGemm g) {
    // K slab: 32 for 64x64 tiles, 64 for 32x32 tiles.  Both operands are widened to float64 once, when they are
    // staged (every staged value is read by 16 threads), so the inner loop is LDS reads and float64 FMAs only.
    constexpr int kF32K = (TS == 32) ? 64 : 32;
    constexpr int EA = TS * kF32K / 256;        // consecutive k one thread stages per row / column (8)
    constexpr int TPR = kF32K / EA;             // threads per staged row
    constexpr int TT = TS / 16;                 // outputs per thread along each side
    static_assert(16 % EA == 0, "the codes a thread expands sit in one packed word");
    __shared__ double As[kF32K][TS + 2];
    __shared__ double Bs[kF32K][TS + 2];

    const int tid = threadIdx.x;
    const int tiles_n = (g.NC + TS - 1) / TS;
    const int64_t m0 = static_cast<int64_t>(blockIdx.x / tiles_n) * TS;
    const int n0 = static_cast<int>(blockIdx.x % tiles_n) * TS;
    const float* __restrict__ X = static_cast<const float*>(g.X);
    const uint32_t* __restrict__ Wq = static_cast<const uint32_t*>(g.Wq);

    // A staging: EA consecutive k of one row; B staging: EA consecutive codes of one output channel
    const int arow = tid / TPR;
    const int akq = (tid % TPR) * EA;
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
    const int bn = n0 + arow;

    float pa[EA];
    uint32_t pw = 0;
    // Branch-free: every lane loads (element 0 when its tap is outside the image or beyond K) and the value is
    // selected afterwards, so the EA loads of a slab are issued back to back instead of one exposed latency each.
    bool okv[EA];       // which of the prefetched values are real (applied when they are staged, so that nothing
    bool wok = false;   // waits for the loads before the slab in between has been multiplied)
    auto fetch = [&](int k0) {
        int64_t idx[EA];
        // (tap, channel) of the first element by division (there is no integer divide in hardware: one pair per
        // slab and thread, not one per element), of the following ones by stepping
        const int kf = k0 + akq;
        int rs = g.plain_gemm ? 0 : kf / g.IC;
        int c = kf - rs * g.IC;
        int r = g.plain_gemm ? 0 : rs / g.S;
        int s_ = rs - r * g.S;
#pragma unroll
        for (int e = 0; e < EA; ++e) {
            int th = ih0 + r * g.dh, tw = iw0 + s_ * g.dw;
            bool ok = kf + e < g.K;
            if (g.divh > 1) { ok = ok && th >= 0 && (th % g.divh) == 0; th /= g.divh; }
            if (g.divw > 1) { ok = ok && tw >= 0 && (tw % g.divw) == 0; tw /= g.divw; }
            ok = ok && static_cast<unsigned>(th) < static_cast<unsigned>(g.IH) &&
                 static_cast<unsigned>(tw) < static_cast<unsigned>(g.IW);
            okv[e] = ok;
            idx[e] = ok ? (pixbase + static_cast<int64_t>(th) * g.IW + tw) * g.xs + c : 0;
            if (++c == g.IC) {
                c = 0;
                if (++s_ == g.S) {
                    s_ = 0;
                    ++r;
                }
            }
        }
#pragma unroll
        for (int e = 0; e < EA; ++e) pa[e] = X[idx[e]];
        const int k = k0 + akq;
        wok = bn < g.NC && k < g.K;
        pw = Wq[wok ? static_cast<int64_t>(bn) * g.wpr + (k >> 4) : 0];
    };
    auto stage = [&](int k0) {
        const int kb = k0 + akq;
#pragma unroll
        for (int e = 0; e < EA; ++e) {
            As[akq + e][arow] = okv[e] ? static_cast<double>(pa[e]) : 0.0;
            const int t = (kb + e) & 15;
            const uint32_t fld = wok ? (pw >> ((t & 1) * 16 + (t >> 1) * 2)) & 3u : 0u;
            Bs[akq + e][arow] = (fld & 1u) ? ((fld & 2u) ? -1.0 : 1.0) : 0.0;
        }
    };

    const int ty = tid >> 4, tx = tid & 15;
    double acc[TT][TT] = {};

    fetch(0);
    for (int k0 = 0; k0 < g.K; k0 += kF32K) {
        stage(k0);
        __syncthreads();
        if (k0 + kF32K < g.K) fetch(k0 + kF32K);        // in flight while this slab is multiplied
#pragma unroll 8
        for (int k = 0; k < kF32K; ++k) {
            double a[TT], b[TT];
#pragma unroll
            for (int i = 0; i < TT; ++i) a[i] = As[k][ty * TT + i];
#pragma unroll
            for (int j = 0; j < TT; ++j) b[j] = Bs[k][tx * TT + j];
#pragma unroll
            for (int i = 0; i < TT; ++i)
#pragma unroll
                for (int j = 0; j < TT; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int j = 0; j < TT; ++j) {
        const int ncol = n0 + tx * TT + j;
        if (ncol >= g.NC) continue;
        const float al = g.alpha[ncol / g.rows_per_group];
        const float sc = g.scale ? g.scale[ncol] : 1.0f;
        const float sf = g.shift ? g.shift[ncol] : 0.0f;
#pragma unroll
        for (int i = 0; i < TT; ++i) {
            const int64_t m = m0 + ty * TT + i;
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
    auto blocks = [&](int ts) { return ((g.M + ts - 1) / ts) * ((g.NC + ts - 1) / ts); };
    const int ts = blocks(64) >= 128 ? 64 : 32;
    const int64_t nb = blocks(ts);
    if (nb <= 0 || nb >= (1LL << 31)) return TWN_ERR_SHAPE;
    if (ts == 64)
        gather_gemm_fp32_kernel<64><<<static_cast<unsigned>(nb), 256, 0, st>>>(g);
    else
        gather_gemm_fp32_kernel<32><<<static_cast<unsigned>(nb), 256, 0, st>>>(g);
    return launch_status();
}

}  // namespace twn
