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
// workgroups.  A thread owns (TS/16)^2 outputs.  Problems that still have few tiles and a long reduction (the
// fully-connected layers of LeNet at batch 64: 32 tiles, 13 slabs each) are split along K over blockIdx.y: every
// range writes its float64 sums to the workspace and a second launch adds them in a fixed order and applies the tail.
#include "twn_kernels.h"

namespace twn {

// SPLIT: blockIdx.y owns `kps` slabs of K and writes raw float64 sums to g.partial ([split][M][NC] doubles)
template <int TS, bool SPLIT>
__global__ __launch_bounds__(256) void gather_gemm_fp32_kernel(const GatherGemm g, int kps) {
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

    const int kbeg = SPLIT ? static_cast<int>(blockIdx.y) * kps * kF32K : 0;
    const int kend = SPLIT ? min(g.K, kbeg + kps * kF32K) : g.K;
    fetch(kbeg);
    for (int k0 = kbeg; k0 < kend; k0 += kF32K) {
        stage(k0);
        __syncthreads();
        if (k0 + kF32K < kend) fetch(k0 + kF32K);        // in flight while this slab is multiplied
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

    if constexpr (SPLIT) {
        double* __restrict__ part = reinterpret_cast<double*>(g.partial) + static_cast<int64_t>(blockIdx.y) * g.M * g.NC;
#pragma unroll
        for (int i = 0; i < TT; ++i) {
            const int64_t m = m0 + ty * TT + i;
#pragma unroll
            for (int j = 0; j < TT; ++j) {
                const int ncol = n0 + tx * TT + j;
                if (m < g.M && ncol < g.NC) part[m * g.NC + ncol] = acc[i][j];
            }
        }
        return;
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

// Sum of the K ranges in a fixed order (float64), then the same tail as the unsplit kernel.
__global__ __launch_bounds__(256) void fp32_splitk_finish_kernel(const GatherGemm g) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t total = g.M * g.NC;
    if (i >= total) return;
    const double* __restrict__ part = reinterpret_cast<const double*>(g.partial);
    double sum = 0.0;
    for (int s = 0; s < g.splits; ++s) sum += part[static_cast<int64_t>(s) * total + i];
    const int64_t m = i / g.NC;
    const int ncol = static_cast<int>(i - m * g.NC);
    const float al = g.alpha[ncol / g.rows_per_group];
    const float sc = g.scale ? g.scale[ncol] : 1.0f;
    const float sf = g.shift ? g.shift[ncol] : 0.0f;
    float v = (static_cast<float>(sum) * al) * sc + sf;
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

// Tile side and K ranges of the float32 path: a pure function of the shapes (the workspace query and the launch
// agree).  Problems with at least 128 tiles of 64x64 run those, unsplit.  Smaller ones are split along K towards
// about 1024 workgroups, every range at least two slabs long, at most 16 ranges; they keep 64x64 tiles (half the
// LDS reads per multiply-add of 32x32 tiles) if that still gives 256 workgroups, else 32x32 tiles.
struct Fp32Plan {
    int ts, kslab, splits, kps;
};
static Fp32Plan fp32_plan(const GatherGemm& g) {
    auto blocks = [&](int ts) { return ((g.M + ts - 1) / ts) * ((g.NC + ts - 1) / ts); };
    auto slabs = [&](int kslab) { return (static_cast<int64_t>(g.K) + kslab - 1) / kslab; };
    Fp32Plan p{64, 32, 1, 0};
    if (blocks(64) >= 128) return p;
    const bool split = env_int("TWN_F32_SPLITK", 1) != 0;
    auto ranges = [&](int64_t tiles, int64_t kt, int* kps) {
        int64_t want = 1024 / tiles;
        if (want > kt / 2) want = kt / 2;
        if (want > 16) want = 16;
        if (want < 2 || !split) {
            *kps = 0;
            return 1;
        }
        *kps = static_cast<int>((kt + want - 1) / want);
        return static_cast<int>((kt + *kps - 1) / *kps);
    };
    int kps64 = 0;
    const int s64 = ranges(blocks(64), slabs(32), &kps64);
    if (split && g.M >= 48 && g.NC >= 48 && blocks(64) * s64 >= 256) {
        p.splits = s64;
        p.kps = kps64;
        return p;
    }
    p.ts = 32;
    p.kslab = 64;
    p.splits = ranges(blocks(32), slabs(64), &p.kps);
    return p;
}

int32_t gather_gemm_fp32_splits(const GatherGemm& g) { return fp32_plan(g).splits; }

int32_t launch_gather_gemm_fp32(const GatherGemm& g, hipStream_t st) {
    const Fp32Plan p = fp32_plan(g);
    const int64_t nb = ((g.M + p.ts - 1) / p.ts) * ((g.NC + p.ts - 1) / p.ts);
    if (nb <= 0 || nb >= (1LL << 31)) return TWN_ERR_SHAPE;
    if (g.splits > 1) {
        if (g.splits != p.splits || !g.partial) return TWN_ERR_WORKSPACE;
        const int64_t total = g.M * g.NC;
        if (total >= (1LL << 31) * 256) return TWN_ERR_SHAPE;
        const dim3 grid(static_cast<unsigned>(nb), static_cast<unsigned>(g.splits));
        if (p.ts == 64)
            gather_gemm_fp32_kernel<64, true><<<grid, 256, 0, st>>>(g, p.kps);
        else
            gather_gemm_fp32_kernel<32, true><<<grid, 256, 0, st>>>(g, p.kps);
        fp32_splitk_finish_kernel<<<static_cast<unsigned>((total + 255) / 256), 256, 0, st>>>(g);
        return launch_status();
    }
    if (p.ts == 64)
        gather_gemm_fp32_kernel<64, false><<<static_cast<unsigned>(nb), 256, 0, st>>>(g, 0);
    else
        gather_gemm_fp32_kernel<32, false><<<static_cast<unsigned>(nb), 256, 0, st>>>(g, 0);
    return launch_status();
}

}  // namespace twn
