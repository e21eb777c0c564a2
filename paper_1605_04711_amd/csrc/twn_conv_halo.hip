// Halo-tiled ternary convolution for stride-1 filters with more than one tap (Eq. 2, Alg. 1 step 8, and
// the backward-data pass of Alg. 1 step 9 for stride-1 layers).
//
// The generic implicit-GEMM kernel fetches a fresh [pixels x 64 channels] slab from L2 for every filter
// tap, so a 3x3 layer moves its activations global -> LDS nine times; that path, not the MFMA pipe, is
// what bounds it.  Here a workgroup owns a spatial patch of output pixels (2^ltn images x 2^lty rows x
// 2^ltx columns = BM pixels) and, per slab of 64 input channels, stages the patch plus its halo ONCE:
// every tap then reads its shifted window of the same LDS data (a lane's A-fragment address is just the
// halo pixel of its row plus a wave-uniform tap offset).  Global -> LDS traffic per 64 channels drops from
// R*S*BM pixel rows to (rows+R-1)*(cols+S-1), about 6x for 3x3 filters.  The 2-bit codes do not pass through
// LDS at all: each lane loads the 32 codes of its output channel and tap (8 bytes, L2-resident) straight
// into registers one tap ahead, which keeps the LDS footprint at two halo stages (about 49 KB for a 128-pixel
// patch) so that three workgroups share a CU.
//
// Pipeline: two stages; the slab after the current one is in flight while all R*S*4 MFMA steps of the
// current one run, so a single s_waitcnt vmcnt(0) + s_barrier per slab hands over.  LDS rows are 128 bytes
// (64 channels) with the 16-byte chunk index XOR-ed by (halo pixel >> 1) & 7, applied by choosing which
// global chunk each lane of a direct-to-LDS load fetches.  Arithmetic, operand roles and the fp32 epilogue
// are those of the generic kernel (codes -> bf16 +-2.0 / 0 in registers, alpha/2 afterwards).
#include <type_traits>

#include "twn_kernels.h"
#include "twn_mfma.h"

namespace twn {

__device__ __attribute__((aligned(16))) const uint32_t kHaloZeroBlock[4] = {0u, 0u, 0u, 0u};

constexpr int kHaloMaxLoads = 14;          // direct-to-LDS activation loads per wave and slab
constexpr int kHaloLdsBudget = 159 * 1024;

struct HaloArgs {
    GatherGemm g;
    int32_t ltx, lty, ltn;       // log2 of the patch: 2^ltn images x 2^lty rows x 2^ltx columns
    int32_t hh, hw, hp;          // halo rows, columns, pixels (= 2^ltn * hh * hw)
    int32_t nla;                 // activation loads per wave and slab = ceil(hp / (8 * waves))
    int32_t tiles_x, tiles_y, tiles_n;
    int32_t batch;
    int32_t iy0, ix0;            // input row / column of halo row / column 0 relative to the patch origin
    int32_t roff, soff;          // halo row of tap r = roff + r*dh, halo column of tap s = soff + s*dw
    FastDivU divHW, divHH, divTN, divTX, divTY;
};

// CS = input channels per slab (64 or 32).  An LDS row is one halo pixel of CS channels (CS*2 bytes, CP = CS/8
// chunks of 16 bytes), a wave-level load covers 64/CP pixels, a tap takes KS = CS/16 MFMA steps, and a lane
// needs CS/2 codes per tap and channel tile (one or two 32-bit words).
template <int BM, int BN, int MI, int CS>
__global__ __launch_bounds__((BM / (32 * MI)) * (BN / 64) * 64, (MI == 4) ? 2 : 3) void conv_halo_kernel(const HaloArgs a) {
    constexpr int WM = BM / (32 * MI), WN = BN / 64, NW = WM * WN;
    constexpr int TM = 32 * MI;         // pixels per wave
    constexpr int NI = 2;
    constexpr int CP = CS / 8, PPL = 64 / CP, KS = CS / 16, ROWB = CS * 2, CW = CS / 32;
    constexpr int LCP = (CP == 8) ? 3 : 2;            // log2(CP)
    static_assert(CS == 64 || CS == 32, "slab width");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const GatherGemm& g = a.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lh = lane >> 5;
    const int RS = g.R * g.S;
    const int stage_bytes = a.nla * NW * 1024;

    // workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tiles
    const uint32_t nb = gridDim.x, b = blockIdx.x;
    const uint32_t q8 = nb >> 3, r8 = nb & 7, xcd = b & 7, idx = b >> 3;
    uint32_t t = (xcd < r8) ? xcd * (q8 + 1) + idx : r8 * (q8 + 1) + (xcd - r8) * q8 + idx;
    // tile -> (image group, patch row, patch column, channel tile), channel tile fastest
    uint32_t u = fdiv_u(t, a.divTN);
    const int n0 = static_cast<int>(t - u * a.tiles_n) * BN;
    t = u;
    u = fdiv_u(t, a.divTX);
    const int x0 = static_cast<int>(t - u * a.tiles_x) << a.ltx;
    t = u;
    u = fdiv_u(t, a.divTY);
    const int y0 = static_cast<int>(t - u * a.tiles_y) << a.lty;
    const int img0 = static_cast<int>(u) << a.ltn;

    const uint16_t* __restrict__ X = static_cast<const uint16_t*>(g.X);
    const uint32_t* __restrict__ Wq = static_cast<const uint32_t*>(g.Wq);
    const void* zero = kHaloZeroBlock;

    // 16-byte chunk c of halo pixel hp sits at chunk position c ^ swz(hp): 16 consecutive pixels then spread
    // one logical chunk over all 64 banks
    auto swz = [](int hp) __attribute__((always_inline)) { return (CP == 8) ? ((hp >> 1) & 7) : ((hp >> 2) & 3); };

    // ---- activation loads: wave-level load i of this wave covers halo pixels (i*NW + wave)*PPL .. +PPL-1 ----
    int32_t pix[kHaloMaxLoads];     // input pixel index of this lane's halo pixel, -1 = outside (zero)
#pragma unroll
    for (int i = 0; i < kHaloMaxLoads; ++i) {
        const uint32_t hpi = static_cast<uint32_t>((i * NW + wave) * PPL + (lane >> LCP));
        const uint32_t t1 = fdiv_u(hpi, a.divHW);
        const int hx = static_cast<int>(hpi - t1 * a.hw);
        const uint32_t nl = fdiv_u(t1, a.divHH);
        const int hy = static_cast<int>(t1 - nl * a.hh);
        const int img = img0 + static_cast<int>(nl);
        const int iy = y0 + a.iy0 + hy, ix = x0 + a.ix0 + hx;
        const bool ok = i < a.nla && hpi < static_cast<uint32_t>(a.hp) && img < a.batch &&
                        static_cast<unsigned>(iy) < static_cast<unsigned>(g.IH) &&
                        static_cast<unsigned>(ix) < static_cast<unsigned>(g.IW);
        pix[i] = ok ? (img * g.IH + iy) * g.IW + ix : -1;
    }

    auto issue = [&](int cs, int stage) __attribute__((always_inline)) {
        unsigned char* sA = smem + stage * stage_bytes;
#pragma unroll
        for (int i = 0; i < kHaloMaxLoads; ++i) {
            if (i < a.nla) {
                // this lane fills chunk position lane % CP of its halo pixel: fetch the logical chunk that lives there
                const int hpi = (i * NW + wave) * PPL + (lane >> LCP);
                const int chunk = (lane & (CP - 1)) ^ swz(hpi);
                const void* src = pix[i] >= 0
                                      ? static_cast<const void*>(X + static_cast<int64_t>(pix[i]) * g.xs + cs * CS + chunk * 8)
                                      : zero;
                dma16(src, sA + (i * NW + wave) * 1024);
            }
        }
    };

    // ---- this lane's rows: halo pixel of output pixel m_local at tap (0,0) with roff = soff = 0 ----
    int hp0[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int ml = wm * TM + mi * 32 + lrow;
        const int xl = ml & ((1 << a.ltx) - 1);
        const int yl = (ml >> a.ltx) & ((1 << a.lty) - 1);
        const int nl = ml >> (a.ltx + a.lty);
        hp0[mi] = (nl * a.hh + yl) * a.hw + xl;
    }

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.0f;

    // ---- packed codes: this lane's output channel of tile ni, the CS/2 codes (CW words) of its k half ----
    const uint32_t* wrow[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int ncol = n0 + wn * 64 + ni * 32 + lrow;
        wrow[ni] = (ncol < g.NC) ? Wq + static_cast<int64_t>(ncol) * g.wpr + CW * lh : nullptr;
    }
    auto load_codes = [&](int cs, int tap, u32x2* dst) __attribute__((always_inline)) {
        const int word = (tap * g.IC + cs * CS) >> 4;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            if (CW == 2) dst[ni] = wrow[ni] ? *reinterpret_cast<const u32x2*>(wrow[ni] + word) : u32x2{0u, 0u};
            else dst[ni] = u32x2{wrow[ni] ? wrow[ni][word] : 0u, 0u};
        }
    };

    const int ncs = g.IC / CS;
    issue(0, 0);
    u32x2 bnext[NI];
    load_codes(0, 0, bnext);
    int stage = 0;
    for (int cs = 0; cs < ncs; ++cs) {
        // slab cs has landed for every wave, and every wave is done with the other stage
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (cs + 1 < ncs) issue(cs + 1, stage ^ 1);

        const unsigned char* sA = smem + stage * stage_bytes;
        int r = 0, s = 0;
        for (int tap = 0; tap < RS; ++tap) {
            const int toff = (a.roff + r * g.dh) * a.hw + (a.soff + s * g.dw);
            u32x2 breg[NI];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) breg[ni] = bnext[ni];
            // the codes of the next tap (or of the next slab's first tap) are fetched one tap ahead
            if (tap + 1 < RS) load_codes(cs, tap + 1, bnext);
            else if (cs + 1 < ncs) load_codes(cs + 1, 0, bnext);
            const unsigned char* rowp[MI];
            int sw[MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int hpm = hp0[mi] + toff;
                rowp[mi] = sA + hpm * ROWB;
                sw[mi] = swz(hpm);
            }
            // lane (row, lh) holds at MFMA step kk the 8 channels of logical chunk lh*KS + kk
            u32x4 afrag[2][MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                afrag[0][mi] = *reinterpret_cast<const u32x4*>(rowp[mi] + (((lh * KS) ^ sw[mi]) << 4));
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                if (kk + 1 < KS) {
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
                        afrag[(kk + 1) & 1][mi] =
                            *reinterpret_cast<const u32x4*>(rowp[mi] + (((lh * KS + kk + 1) ^ sw[mi]) << 4));
                }
                __builtin_amdgcn_sched_barrier(0);
                u32x4 bfrag[NI];
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    // codes of this lane's k half in k order: step kk uses fields 4*kk .. 4*kk+3 of its word(s)
                    const uint32_t word = breg[ni][kk >> 1];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i = (kk & 1) * 4 + e;
                        bfrag[ni][e] = (word << (14 - 2 * i)) & 0xC000C000u;
                    }
                }
                // weights are the MFMA row operand: a lane then owns 4 consecutive output channels of a pixel
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, bfrag[ni]), __builtin_bit_cast(bf16x8, afrag[kk & 1][mi]),
                            acc[mi][ni], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (++s == g.S) {
                s = 0;
                ++r;
            }
        }
        stage ^= 1;
    }

    // ---- epilogue: y = relu?((0.5*alpha*acc)*scale + shift + residual) ----
    // accumulator element e of tile (mi, ni): pixel m_local = wm*TM + mi*32 + lrow,
    // channel n0 + wn*64 + ni*32 + (e>>2)*8 + lh*4 + (e&3)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int ml = wm * TM + mi * 32 + lrow;
        const int ox = x0 + (ml & ((1 << a.ltx) - 1));
        const int oy = y0 + ((ml >> a.ltx) & ((1 << a.lty) - 1));
        const int img = img0 + (ml >> (a.ltx + a.lty));
        if (img >= a.batch || oy >= g.OH || ox >= g.OW) continue;
        const int64_t row = (static_cast<int64_t>(img) * g.OH + oy) * g.OW + ox;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int ncol = n0 + wn * 64 + ni * 32 + q4 * 8 + lh * 4;
                if (ncol >= g.NC) continue;      // NC % 8 == 0 here: a quad is all in or all out
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int c = ncol + e;
                    const float mul = 0.5f * g.alpha[c / g.rows_per_group] * (g.scale ? g.scale[c] : 1.0f);
                    v[e] = acc[mi][ni][q4 * 4 + e] * mul + (g.shift ? g.shift[c] : 0.0f);
                }
                const int64_t off = row * g.ldy + ncol;
                if (g.y_f32) {
                    if (g.residual) {
                        const f32x4 rr = *reinterpret_cast<const f32x4*>(static_cast<const float*>(g.residual) + off);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += rr[e];
                    }
                    if (g.relu) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
                    }
                    *reinterpret_cast<f32x4*>(static_cast<float*>(g.Y) + off) = f32x4{v[0], v[1], v[2], v[3]};
                } else {
                    if (g.residual) {
                        const u32x2 rr = *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(g.residual) + off);
                        v[0] += __uint_as_float(rr[0] << 16);
                        v[1] += __uint_as_float(rr[0] & 0xFFFF0000u);
                        v[2] += __uint_as_float(rr[1] << 16);
                        v[3] += __uint_as_float(rr[1] & 0xFFFF0000u);
                    }
                    if (g.relu) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
                    }
                    u32x2 pk;
                    pk[0] = static_cast<uint32_t>(f32_to_bf16(v[0])) | (static_cast<uint32_t>(f32_to_bf16(v[1])) << 16);
                    pk[1] = static_cast<uint32_t>(f32_to_bf16(v[2])) | (static_cast<uint32_t>(f32_to_bf16(v[3])) << 16);
                    *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(g.Y) + off) = pk;
                }
            }
        }
    }
}

// ---- host side: is the kernel applicable, and with which patch ---------------------------------

static int abs_i(int v) { return v < 0 ? -v : v; }

// Patch of BM = 2^k output pixels (powers of two along batch, rows, columns) that wastes the fewest padded
// pixels and whose halo fits the LDS and load budgets; false if none does.
template <int BM, int BN, int MI, int CS>
static bool halo_plan(const GatherGemm& g, HaloArgs* a) {
    constexpr int NW = (BM / (32 * MI)) * (BN / 64);
    constexpr int PPL = 64 / (CS / 8);      // halo pixels per wave-level load
    if (g.IC % CS != 0) return false;
    int lbm = 0;
    while ((1 << lbm) < BM) ++lbm;
    const int eh = (g.R - 1) * abs_i(g.dh), ew = (g.S - 1) * abs_i(g.dw);
    const int64_t batch = g.M / (static_cast<int64_t>(g.OH) * g.OW);
    int64_t best = -1;
    for (int ltx = lbm; ltx >= 0; --ltx)
        for (int lty = lbm - ltx; lty >= 0; --lty) {
            const int ltn = lbm - ltx - lty;
            const int tx = 1 << ltx, ty = 1 << lty, tn = 1 << ltn;
            // a patch dimension beyond twice the image only adds padding
            if ((tx >> 1) >= g.OW && ltx > 0) continue;
            if ((ty >> 1) >= g.OH && lty > 0) continue;
            if ((tn >> 1) >= batch && ltn > 0) continue;
            const int hh = ty + eh, hw = tx + ew;
            const int64_t hp = static_cast<int64_t>(tn) * hh * hw;
            const int64_t nla = (hp + PPL * NW - 1) / (PPL * NW);
            if (nla > kHaloMaxLoads) continue;
            const int64_t stage = nla * NW * 1024;
            if (2 * stage > kHaloLdsBudget) continue;
            const int64_t tiles = ((g.OW + tx - 1) / tx) * static_cast<int64_t>((g.OH + ty - 1) / ty) * ((batch + tn - 1) / tn);
            // fewest padded pixels first, then the smallest halo
            const int64_t cost = tiles * 4096 + hp;
            if (best < 0 || cost < best) {
                best = cost;
                a->ltx = ltx; a->lty = lty; a->ltn = ltn;
                a->hh = hh; a->hw = hw; a->hp = static_cast<int32_t>(hp);
                a->nla = static_cast<int32_t>(nla);
                a->tiles_x = (g.OW + tx - 1) / tx;
                a->tiles_y = (g.OH + ty - 1) / ty;
            }
        }
    if (best < 0) return false;
    a->g = g;
    a->batch = static_cast<int32_t>(batch);
    a->tiles_n = (g.NC + BN - 1) / BN;
    const int rmin = (g.dh < 0) ? (g.R - 1) * g.dh : 0, smin = (g.dw < 0) ? (g.S - 1) * g.dw : 0;
    a->iy0 = -g.ph + rmin;
    a->ix0 = -g.pw + smin;
    a->roff = -rmin;
    a->soff = -smin;
    a->divHW = make_fastdiv_u(a->hw);
    a->divHH = make_fastdiv_u(a->hh);
    a->divTN = make_fastdiv_u(a->tiles_n);
    a->divTX = make_fastdiv_u(a->tiles_x);
    a->divTY = make_fastdiv_u(a->tiles_y);
    return true;
}

static int64_t halo_blocks(const HaloArgs& a) {
    const int64_t groups = (a.batch + (1 << a.ltn) - 1) >> a.ltn;
    return groups * a.tiles_y * a.tiles_x * a.tiles_n;
}

template <int BM, int BN, int MI, int CS>
static int32_t launch_halo(const HaloArgs& a, hipStream_t st) {
    constexpr int NW = (BM / (32 * MI)) * (BN / 64);
    const int smem = 2 * a.nla * NW * 1024;
    const int64_t blocks = halo_blocks(a);
    if (blocks <= 0 || blocks >= (1LL << 31)) return TWN_ERR_SHAPE;
    static bool allowed = false;
    auto k = conv_halo_kernel<BM, BN, MI, CS>;
    if (!allowed) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                kHaloLdsBudget) != hipSuccess) return TWN_ERR_HIP;
        allowed = true;
    }
    k<<<dim3(static_cast<unsigned>(blocks)), dim3(64 * NW), smem, st>>>(a);
    return launch_status();
}

// Stride-1 layers with several taps, channel counts in whole 64-wide slabs, no split over K.
bool conv_halo_applicable(const GatherGemm& g) {
    // Off unless TWN_HALO=1: with compiler-placed LDS waits and 64x64 wave tiles this first version only
    // matches the generic kernel (see the measurements in the design notes); it is kept parity-tested.
    if (env_int("TWN_HALO", 0) == 0) return false;
    if (g.plain_gemm || g.chunk_gather || g.splits > 1) return false;
    if (g.R * g.S <= 1 || g.sh != 1 || g.sw != 1 || g.divh != 1 || g.divw != 1) return false;
    if (g.IC % 64 != 0 || g.xs % 8 != 0 || g.NC % 8 != 0 || g.ldy % 4 != 0) return false;
    if (g.M % (static_cast<int64_t>(g.OH) * g.OW) != 0) return false;
    if (static_cast<int64_t>(g.M / (static_cast<int64_t>(g.OH) * g.OW)) * g.IH * g.IW >= (1LL << 31)) return false;
    HaloArgs a;
    return halo_plan<128, 128, 2, 64>(g, &a);
}

int32_t launch_conv_halo(const GatherGemm& g, hipStream_t st) {
    HaloArgs a;
    if (g.NC <= 64) {
        // 64 output channels: four waves of 32 pixels each
        if (!halo_plan<128, 64, 1, 64>(g, &a)) return TWN_ERR_UNSUPPORTED;
        return launch_halo<128, 64, 1, 64>(a, st);
    }
    // TWN_HALO_SHAPE=1: 256-pixel patches, 128-pixel wave tiles (four MFMAs per expanded code fragment) and
    // 32-channel slabs (two halo stages stay near 48 KB, two workgroups per CU); measured slower than the
    // 128-pixel shape on every benchmark layer except the largest grids, where it ties
    if (env_int("TWN_HALO_SHAPE", 0) == 1 && halo_plan<256, 128, 4, 32>(g, &a)) return launch_halo<256, 128, 4, 32>(a, st);
    if (!halo_plan<128, 128, 2, 64>(g, &a)) return TWN_ERR_UNSUPPORTED;
    return launch_halo<128, 128, 2, 64>(a, st);
}

}  // namespace twn
