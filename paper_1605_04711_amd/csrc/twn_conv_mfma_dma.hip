// Multi-stage implicit-GEMM ternary convolution / inner product on gfx950
// (Eq. 2, Alg. 1 step 8; also the backward-data pass of Alg. 1 step 9).
//
// Same arithmetic as the register-staged kernel (bf16 activations as the MFMA A
// operand, 2-bit codes expanded in registers to +-2.0 / 0 as the B operand,
// alpha/2 applied in the fp32 epilogue), but every tile travels global -> LDS
// by direct 16-byte LDS loads (global_load_lds_dwordx4), STAGES slabs deep:
//   * per K slab of 64 a workgroup stages BM rows x 128 bytes of activations
//     (16-byte chunks XOR-swizzled by (row >> 1) & 7: the swizzle is applied by
//     choosing which global chunk each lane fetches, because a direct LDS load
//     always writes lane j of a wave at byte 16*j of its 1 KB destination) and
//     BN x 16 bytes of packed codes (64 codes of each output channel);
//   * loads for slab kt+STAGES-1 are issued while slab kt is multiplied; one
//     s_waitcnt vmcnt(N) + s_barrier per slab hands a landed slab to all waves;
//   * lanes outside the image / beyond M, N or K fetch from a 16-byte zero
//     block instead, so padding costs no branches and slabs past the end of K
//     are harmless zero loads that keep the outstanding-load count constant.
#include "twn_agpr_tiles.h"
#include <mutex>

#include "twn_kernels.h"
#include "twn_lds_asm.h"
#include "twn_mfma.h"

namespace twn {

__device__ __attribute__((aligned(16))) const uint32_t kZeroBlock[4] = {0u, 0u, 0u, 0u};

#ifdef TWN_TRACE
// development build only: per-workgroup phase timestamps (shader clock) written to a buffer set from the host
__device__ uint64_t* g_trace = nullptr;
#define TWN_TRACE_POINT(slot)                                                                         \
    do {                                                                                              \
        if (g_trace && threadIdx.x == 0) g_trace[static_cast<size_t>(blockIdx.x) * 8 + (slot)] = __builtin_readcyclecounter(); \
    } while (0)
#else
#define TWN_TRACE_POINT(slot) do {} while (0)
#endif

struct DmaArgs {
    GatherGemm g;
    FastDivU divIC, divS;
    // 1: loads go through buffer descriptors (x_bytes, w_bytes < 2 GiB; plain GEMM with K % 64 == 0, or a
    // convolution without tap division whose channel count is a multiple of 64, so that a slab is one tap)
    int32_t use_buf;
    uint32_t x_bytes, w_bytes;
    FastDivU divUV, divV;       // output row remap (g.orU > 0): row -> (image, u, v)
    FastDivU divOW, divOH;      // GEMM row -> (image, oh, ow) of the gather's output grid (M < 2^31)
};

// Row of Y that GEMM row m is written to (see GatherGemm::orU).
__device__ __forceinline__ int64_t out_row(const GatherGemm& g, const FastDivU& divUV, const FastDivU& divV, int64_t m) {
    if (g.orU == 0) return m;
    const uint32_t mu = static_cast<uint32_t>(m);
    const uint32_t n = fdiv_u(mu, divUV);
    const uint32_t rem = mu - n * static_cast<uint32_t>(g.orU * g.orV);
    const uint32_t u = fdiv_u(rem, divV);
    const uint32_t v = rem - u * static_cast<uint32_t>(g.orV);
    return (static_cast<int64_t>(n) * g.orH + g.ora + g.orsh * static_cast<int>(u)) * g.orW + g.orb + g.orsw * static_cast<int>(v);
}

// workgroups per CU the register allocation should allow: two waves per SIMD where LDS permits
constexpr int dma_min_blocks(int nw, int smem) {
    int by_waves = 8 / nw, by_lds = (160 * 1024) / smem;
    int b = by_waves < by_lds ? by_waves : by_lds;
    return b < 1 ? 1 : b;
}

// The kernel proper: workgroup `b` of `nb` of problem `a` (`by`: the K range of a split-K launch).
template <int BM, int BN, int WM, int WN, int STAGES, bool GEMM, bool SPLITK, bool BUF>
__device__ __forceinline__ void gather_gemm_dma_body(const DmaArgs& a, const uint32_t nb, const uint32_t b, const uint32_t by) {
    constexpr int NW = WM * WN;                    // waves per workgroup
    constexpr int NT = 64 * NW;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int NLOAD = BM / (8 * NW);           // 1 KB (8 rows) per wave-level load
    constexpr int A_BYTES = BM * 128;
    constexpr int B_BYTES = BN * 16;
    constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int PD = STAGES - 1;                 // slabs in flight ahead of the one being multiplied
    constexpr int PER_STAGE = NLOAD + 1;           // vector-memory loads per wave per slab
    // 16 accumulator tiles per wave fill the accumulation registers exactly: they are then pinned by hand
    constexpr bool PINNED = (MI * NI == 16);
    // epilogue staging: EPI_CH channels of every pixel row of a wave's tile at a time (64 when LDS allows)
    constexpr int EPI_CH = (TN % 64 == 0 && NW * TM * 144 + 2 * BN * 4 <= STAGES * STAGE_BYTES) ? 64 : 32;
    constexpr int EPI_ROW = EPI_CH * 2 + 16;       // bytes per staged pixel row (pad keeps 16-byte reads conflict-free)
    constexpr int EPI_NI = EPI_CH / 32;            // 32-channel MFMA tiles per staged chunk
    constexpr int EPI_STAGE_BYTES = NW * TM * EPI_ROW;
    static_assert(BM % (8 * NW) == 0 && BN % 64 == 0 && BN <= 64 * NW && TN % 32 == 0 && TM % 32 == 0, "tile shape");
    static_assert(STAGES >= 3, "the mid-slab hand-over needs two slabs in flight");
    static_assert(EPI_STAGE_BYTES + 2 * BN * 4 <= STAGES * STAGE_BYTES, "epilogue staging must fit in the pipeline LDS");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    TWN_TRACE_POINT(0);
#ifdef TWN_TRACE
    if (g_trace && threadIdx.x == 0) {
        uint32_t hw, xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        g_trace[static_cast<size_t>(blockIdx.x) * 8 + 6] = (static_cast<uint64_t>(xcc) << 32) | hw;
        g_trace[static_cast<size_t>(blockIdx.x) * 8 + 7] = wall_clock64();
    }
#endif
    const GatherGemm& g = a.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lh = lane >> 5;

    // workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tiles
    const uint32_t q = nb >> 3, r = nb & 7, xcd = b & 7, idx = b >> 3;
    const uint32_t t = (xcd < r) ? xcd * (q + 1) + idx : r * (q + 1) + (xcd - r) * q + idx;
    const uint32_t tiles_n = (g.NC + BN - 1) / BN;
    const int64_t m0 = static_cast<int64_t>(t / tiles_n) * BM;
    const int n0 = static_cast<int>(t % tiles_n) * BN;

    const uint16_t* __restrict__ X = static_cast<const uint16_t*>(g.X);
    const uint32_t* __restrict__ Wq = static_cast<const uint32_t*>(g.Wq);
    const void* zero = kZeroBlock;

    // ---- A loads: wave-level load i of this wave covers rows (i*NW + wave)*8 .. +7 ----
    // LDS row r keeps logical chunk c at position c ^ ((r >> 1) & 7): with 64 banks, 16 consecutive rows of
    // one logical chunk then fall in 16 different 16-byte bank groups (conflict-free ds_read_b128)
    const int kc = (lane & 7) ^ ((wave & 1) * 4 + ((lane >> 4) & 3));   // logical chunk this lane fetches
    int64_t abase[NLOAD];                              // GEMM: element offset of the row; conv: pixel base
    int64_t off0[NLOAD];                               // conv: element offset of tap (0,0), may be negative
    int ih0[NLOAD], iw0[NLOAD];
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int row = (i * NW + wave) * 8 + (lane >> 3);
        const int64_t m = m0 + row;
        if (m < g.M) {
            if (GEMM) {
                abase[i] = m * g.xs;
                ih0[i] = 0;
                iw0[i] = 0;
            } else {
                // M < 2^31: exact 32-bit division by multiplication instead of 64-bit divisions
                const uint32_t mu = static_cast<uint32_t>(m);
                const uint32_t tt = fdiv_u(mu, a.divOW);
                const int ow = static_cast<int>(mu - tt * static_cast<uint32_t>(g.OW));
                const uint32_t img = fdiv_u(tt, a.divOH);
                const int oh = static_cast<int>(tt - img * static_cast<uint32_t>(g.OH));
                abase[i] = static_cast<int64_t>(img) * (g.IH * g.IW);
                ih0[i] = oh * g.sh - g.ph;
                iw0[i] = ow * g.sw - g.pw;
            }
        } else {
            abase[i] = 0;
            ih0[i] = -(1 << 28);
            iw0[i] = -(1 << 28);
        }
        off0[i] = (abase[i] + static_cast<int64_t>(ih0[i]) * g.IW + iw0[i]) * g.xs;
    }
    const bool undivided = (g.divh == 1 && g.divw == 1);   // everything except strided backward-data
    // buffer-descriptor path: per-lane byte offsets that stay fixed for the whole K loop
    constexpr bool use_buf = BUF;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(X, a.x_bytes), rw = make_rsrc(Wq, a.w_bytes);
    uint32_t voffA[NLOAD];      // GEMM: the row's offset (or kBufOutside); convolution: offset of tap (0,0), any sign
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int64_t bytes = ((GEMM ? abase[i] : off0[i]) + kc * 8) * 2;
        voffA[i] = (GEMM && ih0[i] != 0) ? kBufOutside : static_cast<uint32_t>(static_cast<int32_t>(bytes));
    }
    // ---- B load: this wave stages the packed codes of 64 output channels (one lane per channel) ----
    const int brow = (wave * 64) % BN + lane;
    const int bcol = n0 + brow;
    const uint32_t* bsrc = (bcol < g.NC) ? Wq + static_cast<int64_t>(bcol) * g.wpr : nullptr;
    const uint32_t voffB = (bcol < g.NC) ? static_cast<uint32_t>(bcol) * static_cast<uint32_t>(g.wpr) * 4u : kBufOutside;

    // K slabs handled by this workgroup: all of them, or one range of a split-K launch (blockIdx.y)
    const int KT_all = (g.K + 63) / 64;
    const int kps = SPLITK ? (KT_all + g.splits - 1) / g.splits : KT_all;
    const int kt_begin = SPLITK ? static_cast<int>(by) * kps : 0;
    const int KT = (kt_begin + kps < KT_all) ? kt_begin + kps : KT_all;      // end of this range

    auto tap_coord = [&](int base, int tap, int step, int div, int limit, int& out) __attribute__((always_inline)) -> bool {
        int v = base + tap * step;
        if (div > 1) {
            if (v < 0 || (v % div) != 0) return false;
            v /= div;
        }
        out = v;
        return static_cast<unsigned>(v) < static_cast<unsigned>(limit);
    };

    // Loads of one slab, cut into pieces so that the main loop can spread them between MFMAs:
    // issue_setup fixes the slab (per-lane k offset, tap), issue_load<I> issues load I of NLOAD + 1
    // (the last one stages the packed codes).
    struct {
        unsigned char* sbase;
        int kt, k, c, rr, ss, dth, dtw;
        int64_t delta;
        bool kok;
        int ktc;            // buffer path: slab index clamped to the range (slabs past the end re-read the last one)
        int32_t delta_b;    // buffer path, convolution: byte offset of this slab's tap and channel base (wave-uniform)
        // buffer path, convolution: channel base and tap of the NEXT slab to issue (issue_setup is called for
        // consecutive slabs, so these run as counters instead of being divided out of the slab index)
        int nc0, nss, nrr;
    } si;
    if constexpr (use_buf && !GEMM) {
        const uint32_t kb = static_cast<uint32_t>(kt_begin) * 64u;
        const uint32_t rs = fdiv_u(kb, a.divIC);
        si.nc0 = static_cast<int>(kb - rs * g.IC);
        si.nrr = static_cast<int>(fdiv_u(rs, a.divS));
        si.nss = static_cast<int>(rs) - si.nrr * g.S;
    }
    const int32_t strR = g.dh * g.IW * static_cast<int>(g.xs) * 2, strS = g.dw * static_cast<int>(g.xs) * 2;
    auto issue_setup = [&](int kt, int stage) __attribute__((always_inline)) {
        si.sbase = smem + stage * STAGE_BYTES;
        si.kt = kt;
        if constexpr (use_buf) {
            // everything here is wave-uniform: scalar instructions only
            si.ktc = (kt < KT) ? kt : KT - 1;
            if (!GEMM) {
                si.delta_b = si.nrr * strR + si.nss * strS + si.nc0 * 2;
                si.dth = si.nrr * g.dh;
                si.dtw = si.nss * g.dw;
                // a slab past the end re-reads the last one: the counters stop there
                if (kt < KT - 1) {
                    si.nc0 += 64;
                    if (si.nc0 == g.IC) {
                        si.nc0 = 0;
                        if (++si.nss == g.S) {
                            si.nss = 0;
                            ++si.nrr;
                        }
                    }
                }
            }
            return;
        }
        si.k = kt * 64 + kc * 8;
        si.kok = (kt < KT) && (si.k < g.K);
        if (!GEMM) {
            const uint32_t rs = fdiv_u(static_cast<uint32_t>(si.k), a.divIC);
            si.c = si.k - static_cast<int>(rs) * g.IC;
            si.rr = static_cast<int>(fdiv_u(rs, a.divS));
            si.ss = static_cast<int>(rs) - si.rr * g.S;
            // one tap offset per slab for this lane; per row: two bounds tests and one 64-bit add
            si.dth = si.rr * g.dh;
            si.dtw = si.ss * g.dw;
            si.delta = (static_cast<int64_t>(si.dth) * g.IW + si.dtw) * g.xs + si.c;
        }
    };
    auto issue_load = [&](auto i_tag) __attribute__((always_inline)) {
        constexpr int i = decltype(i_tag)::value;
        if constexpr (use_buf) {
            if constexpr (i == NLOAD) {
                buf_dma16(rw, voffB, static_cast<uint32_t>(si.ktc) * 16u, si.sbase + A_BYTES + ((wave * 64) % BN) * 16);
            } else if (GEMM) {
                buf_dma16(rx, voffA[i], static_cast<uint32_t>(si.ktc) * 128u, si.sbase + (i * NW + wave) * 1024);
            } else {
                const bool ok = (static_cast<unsigned>(ih0[i] + si.dth) < static_cast<unsigned>(g.IH)) &
                                (static_cast<unsigned>(iw0[i] + si.dtw) < static_cast<unsigned>(g.IW));
                buf_dma16(rx, ok ? voffA[i] + static_cast<uint32_t>(si.delta_b) : kBufOutside, 0u,
                          si.sbase + (i * NW + wave) * 1024);
            }
            return;
        }
        if constexpr (i == NLOAD) {
            const void* bs = (bsrc && si.kt < KT) ? static_cast<const void*>(bsrc + si.kt * 4) : zero;
            dma16(bs, si.sbase + A_BYTES + ((wave * 64) % BN) * 16);
        } else {
            const void* src;
            if (GEMM) {
                src = (si.kok && ih0[i] == 0) ? static_cast<const void*>(X + abase[i] + si.k) : zero;
            } else if (undivided) {
                const bool ok = si.kok && static_cast<unsigned>(ih0[i] + si.dth) < static_cast<unsigned>(g.IH) &&
                                static_cast<unsigned>(iw0[i] + si.dtw) < static_cast<unsigned>(g.IW);
                src = ok ? static_cast<const void*>(X + off0[i] + si.delta) : zero;
            } else {
                int th, tw;
                bool ok = tap_coord(ih0[i], si.rr, g.dh, g.divh, g.IH, th);
                ok = tap_coord(iw0[i], si.ss, g.dw, g.divw, g.IW, tw) && ok && si.kok;
                src = ok ? static_cast<const void*>(X + (abase[i] + static_cast<int64_t>(th) * g.IW + tw) * g.xs + si.c)
                         : zero;
            }
            dma16(src, si.sbase + (i * NW + wave) * 1024);
        }
    };
    auto issue = [&](int kt, int stage) __attribute__((always_inline)) {
        issue_setup(kt, stage);
        static_for<NLOAD + 1>(issue_load);
    };

    f32x16 acc[PINNED ? 1 : MI][PINNED ? 1 : NI];
    if constexpr (PINNED) {
        static_for<16>([&](auto j_tag) __attribute__((always_inline)) { AgprTile<decltype(j_tag)::value>::zero(); });
    } else {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.0f;
    }
    // accumulator tile (mi, ni) as a value, for the epilogue
    auto acc_tile = [&](int mi, int ni) __attribute__((always_inline)) -> f32x16 {
        if constexpr (PINNED) {
            return agpr_read(mi * NI + ni);
        } else {
            return acc[mi][ni];
        }
    };

    // ---- software pipeline ---------------------------------------------------------------------
    // Slab kt lives in stage kt % STAGES and is multiplied in four MFMA steps kk = 0..3 of MI*NI MFMAs.
    // Everything that is not an MFMA is cut into small pieces and placed BETWEEN the MFMAs of a step, so
    // that a wave never has an MFMA-free stretch (two waves share a SIMD's matrix pipe and tend to fall
    // into step with each other, so such stretches are not filled by the other wave):
    //   * the LDS reads of the next step's activation fragments (one step ahead, other register set),
    //   * the expansion of the next step's packed codes to bf16 {0, +2, -2},
    //   * in steps 2 and 3, the direct-to-LDS loads of slab kt+PD and the read of slab kt+1's codes.
    // The hand-over point sits between steps 1 and 2: wait until slab kt+1 has landed, barrier; the stage
    // of slab kt-1 is then free for slab kt+PD and slab kt+1 may be read.
    static_assert(MI <= 8 && NI <= 4, "fragment reads use immediate offsets");
    // LDS byte address of the dynamic array (the low 32 bits of its generic address are the LDS offset)
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) unsigned char*)smem));
    // per-lane byte offsets inside a stage; the swizzle term does not depend on mi because TM % 32 == 0
    uint32_t aoff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        aoff[kk] = (wm * TM + lrow) * 128 + (((lh * 4 + kk) ^ ((lrow >> 1) & 7)) * 16);
    const uint32_t boff = A_BYTES + (wn * TN + lrow) * 16 + lh * 8;

    u32x2 breg[2][NI];      // packed codes of the slab being multiplied / of the next slab
    u32x4 afrag[2][MI];     // activation fragments of step kk in set kk & 1
    u32x4 bfrag[2][NI];     // expanded codes of step kk in set kk & 1

    // code field i of every 32-bit half lands in bits [14,15] of a bf16: 0 / +2.0 / -2.0.  The field is
    // masked first (masks held in scalar registers), then shifted: the intermediate is mostly zero bits.
    uint32_t kmask[8];
    kmask[0] = sgpr_const<static_cast<int>(0xC000C000u >> 14)>();
    kmask[1] = sgpr_const<static_cast<int>(0xC000C000u >> 12)>();
    kmask[2] = sgpr_const<static_cast<int>(0xC000C000u >> 10)>();
    kmask[3] = sgpr_const<static_cast<int>(0xC000C000u >> 8)>();
    kmask[4] = sgpr_const<static_cast<int>(0xC000C000u >> 6)>();
    kmask[5] = sgpr_const<static_cast<int>(0xC000C000u >> 4)>();
    kmask[6] = sgpr_const<static_cast<int>(0xC000C000u >> 2)>();
    kmask[7] = sgpr_const<static_cast<int>(0xC000C000u)>();
    auto expand = [&](auto kk_tag, auto ni_tag, auto e_tag, const u32x2* br, u32x4* out) __attribute__((always_inline)) {
        constexpr int kk = decltype(kk_tag)::value, ni = decltype(ni_tag)::value, e = decltype(e_tag)::value;
        constexpr int i = (kk & 1) * 4 + e;
        out[ni][e] = (br[ni][kk >> 1] & kmask[i]) << (14 - 2 * i);
    };

    // One MFMA step.  Weights are the MFMA row operand, activations the column operand: a lane then owns
    // 4 consecutive output channels of one pixel per accumulator quad.
    auto step = [&](auto kk_tag, auto cur_tag, int kt, int stage, int next, int fill) __attribute__((always_inline)) {
        constexpr int KK = decltype(kk_tag)::value;
        constexpr int CUR = decltype(cur_tag)::value;
        constexpr int NM = MI * NI;
        constexpr int SET = KK & 1, NSET = SET ^ 1;
        constexpr int KN = (KK + 1) & 3;                         // the step being prepared
        constexpr int BSRC = (KK == 3) ? (CUR ^ 1) : CUR;        // its codes: next slab's after the last step
        constexpr int HALF = (NLOAD + 2) / 2;                    // loads issued in step 2, the rest in step 3
        constexpr int G0 = (KK == 2) ? 0 : HALF;
        constexpr int P_RA = MI;                                 // pieces: fragment reads,
        constexpr int P_RB = (KK == 2) ? 1 : 0;                  //   codes of the next slab,
        constexpr int P_D = 4 * NI;                              //   code expansion,
        constexpr int P_G = (KK == 2) ? HALF : (KK == 3) ? NLOAD + 1 - HALF : 0;   //   global loads
        constexpr int P = P_RA + P_RB + P_D + P_G;
        const uint32_t a_addr = lds_base + ((KK == 3) ? next : stage) * STAGE_BYTES + aoff[KN];
        auto piece = [&](auto p_tag) __attribute__((always_inline)) {
            constexpr int p = decltype(p_tag)::value;
            if constexpr (p < P_RA) {
                lds_read128<p * 32 * 128>(afrag[NSET][p], a_addr);
            } else if constexpr (p < P_RA + P_RB) {
                lds_read64_n<NI, 32 * 16>(breg[CUR ^ 1], lds_base + next * STAGE_BYTES + boff);
            } else if constexpr (p < P_RA + P_RB + P_D) {
                constexpr int q = p - P_RA - P_RB;
                expand(std::integral_constant<int, KN>{}, std::integral_constant<int, q / 4>{},
                       std::integral_constant<int, q % 4>{}, breg[BSRC], bfrag[NSET]);
            } else {
                constexpr int gi = G0 + p - (P_RA + P_RB + P_D);
                if constexpr (gi == 0) issue_setup(kt + PD, fill);
                issue_load(std::integral_constant<int, gi>{});
            }
        };
        static_for<NM>([&](auto j_tag) __attribute__((always_inline)) {
            constexpr int j = decltype(j_tag)::value;
            constexpr int mi = j / NI, ni = j % NI;
            if constexpr (PINNED) {
                AgprTile<j>::mfma(bfrag[SET][ni], afrag[SET][mi]);
            } else {
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfrag[SET][ni]),
                                                                      __builtin_bit_cast(bf16x8, afrag[SET][mi]),
                                                                      acc[mi][ni], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            static_for<P>([&](auto p_tag) __attribute__((always_inline)) {
                constexpr int p = decltype(p_tag)::value;
                if constexpr (p * NM / P == j) piece(p_tag);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        // everything read during this step is needed by the next one
        lds_wait<0>();
        lds_ready<MI>(afrag[NSET]);
        if constexpr (KK == 2) lds_ready<NI>(breg[CUR ^ 1]);
        __builtin_amdgcn_sched_barrier(0);
    };

    // prologue: PD slabs in flight, the first one landed and visible to every wave
#pragma unroll
    for (int s = 0; s < PD; ++s) issue(kt_begin + s, s);
    TWN_TRACE_POINT(1);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm((PD - 1) * PER_STAGE));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    TWN_TRACE_POINT(2);
    lds_read64_n<NI, 32 * 16>(breg[0], lds_base + boff);
    lds_read128_n<MI, 32 * 128>(afrag[0], lds_base + aoff[0]);
    lds_wait<0>();
    lds_ready<NI>(breg[0]);
    lds_ready<MI>(afrag[0]);
    static_for<4 * NI>([&](auto q_tag) __attribute__((always_inline)) {
        constexpr int q = decltype(q_tag)::value;
        expand(std::integral_constant<int, 0>{}, std::integral_constant<int, q / 4>{},
               std::integral_constant<int, q % 4>{}, breg[0], bfrag[0]);
    });

    int stage = 0;          // stage of the slab being multiplied
    int fill = PD % STAGES; // stage that slab kt + PD goes to
    // one slab; CUR selects the register set holding this slab's packed codes
    auto slab = [&](int kt, auto cur_tag) __attribute__((always_inline)) {
        const int next = (stage + 1 == STAGES) ? 0 : stage + 1;
        step(std::integral_constant<int, 0>{}, cur_tag, kt, stage, next, fill);
        step(std::integral_constant<int, 1>{}, cur_tag, kt, stage, next, fill);
        // hand-over: slab kt+1 landed (the PD-2 younger slabs may stay in flight), stage of slab kt-1 is free
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((PD - 2) * PER_STAGE));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        step(std::integral_constant<int, 2>{}, cur_tag, kt, stage, next, fill);
        step(std::integral_constant<int, 3>{}, cur_tag, kt, stage, next, fill);
        stage = next;
        fill = (fill + 1 == STAGES) ? 0 : fill + 1;
    };
    for (int kt = kt_begin; kt < KT; kt += 2) {
        slab(kt, std::integral_constant<int, 0>{});
        if (kt + 1 < KT) slab(kt + 1, std::integral_constant<int, 1>{});
    }

    // the trailing zero loads still target LDS: drain them in every wave before LDS is reused
    TWN_TRACE_POINT(3);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    TWN_TRACE_POINT(4);
    if constexpr (PINNED) agpr_settle();

    if (SPLITK) {
        // raw fp32 partial sums; alpha, scale, shift, residual and ReLU are applied by the reduction kernel
        float* part = g.partial + static_cast<int64_t>(by) * g.M * g.NC;
        const bool v4 = (g.NC % 4 == 0);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int64_t m = m0 + wm * TM + mi * 32 + lrow;
            if (m >= g.M) continue;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const f32x16 t = acc_tile(mi, ni);
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int ncol = n0 + wn * TN + ni * 32 + q4 * 8 + lh * 4;
                    float* dst = part + m * g.NC + ncol;
                    if (v4 && ncol < g.NC) {
                        *reinterpret_cast<f32x4*>(dst) = f32x4{t[q4 * 4], t[q4 * 4 + 1], t[q4 * 4 + 2], t[q4 * 4 + 3]};
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (ncol + e < g.NC) dst[e] = t[q4 * 4 + e];
                    }
                }
            }
        }
        return;
    }

    // ---- epilogue: y = relu?((alpha*acc)*scale + shift + residual) ----
    // accumulator element e of tile (mi, ni) in this lane:
    //   pixel   m = wm*TM + mi*32 + lrow
    //   channel n = wn*TN + ni*32 + (e>>2)*8 + lh*4 + (e&3)
    float* colmul = reinterpret_cast<float*>(smem + EPI_STAGE_BYTES);   // [BN] 0.5*alpha*scale
    float* coladd = colmul + BN;                                        // [BN] shift
    for (int i = tid; i < BN; i += NT) {
        const int ncol = n0 + i;
        float mul = 0.0f, add = 0.0f;
        if (ncol < g.NC) {
            const int ag = (g.rows_per_group >= g.NC) ? 0 : ncol / g.rows_per_group;
            mul = 0.5f * g.alpha[ag] * (g.scale ? g.scale[ncol] : 1.0f);   // codes were +-2
            add = g.shift ? g.shift[ncol] : 0.0f;
        }
        colmul[i] = mul;
        coladd[i] = add;
    }
    __syncthreads();

    const bool vec_store = !g.y_f32 && (g.NC % 8 == 0) && (g.ldy % 8 == 0);
    if (vec_store) {
        // bf16 output: finish each value in fp32, round once, transpose 64-channel chunks through
        // LDS (this wave's own region) and write 16 bytes per lane, 64-128 contiguous bytes per pixel
        unsigned char* stg = smem + wave * (TM * EPI_ROW);
        const uint16_t* res = static_cast<const uint16_t*>(g.residual);
        uint16_t* Yb = static_cast<uint16_t*>(g.Y);
#pragma unroll
        for (int nc = 0; nc < NI / EPI_NI; ++nc) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int64_t m = m0 + wm * TM + mi * 32 + lrow;
#pragma unroll
                for (int nh = 0; nh < EPI_NI; ++nh) {
                    const int ni = nc * EPI_NI + nh;
                    const f32x16 t = acc_tile(mi, ni);
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const int nl = wn * TN + ni * 32 + q4 * 8 + lh * 4;     // column within the block tile
                        const f32x4 mul = *reinterpret_cast<const f32x4*>(colmul + nl);
                        const f32x4 add = *reinterpret_cast<const f32x4*>(coladd + nl);
                        float v[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = t[q4 * 4 + e] * mul[e] + add[e];
                        if (res && m < g.M && n0 + nl < g.NC) {
                            const u32x2 rr = *reinterpret_cast<const u32x2*>(res + out_row(g, a.divUV, a.divV, m) * g.ldy + n0 + nl);
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
                        pk[0] = pack_bf16x2(v[0], v[1]);
                        pk[1] = pack_bf16x2(v[2], v[3]);
                        *reinterpret_cast<u32x2*>(stg + (mi * 32 + lrow) * EPI_ROW + (nh * 32 + q4 * 8 + lh * 4) * 2) = pk;
                    }
                }
            }
            // same wave wrote and reads: LDS executes a wave's operations in order
            constexpr int LPR = EPI_CH / 8;          // lanes per staged row (16 bytes each)
#pragma unroll
            for (int it = 0; it < TM * LPR / 64; ++it) {
                const int row = it * (64 / LPR) + lane / LPR;
                const int c16 = lane % LPR;
                const u32x4 val = *reinterpret_cast<const u32x4*>(stg + row * EPI_ROW + c16 * 16);
                const int64_t m = m0 + wm * TM + row;
                const int ncol = n0 + wn * TN + nc * EPI_CH + c16 * 8;
                if (m < g.M && ncol < g.NC) store16_through(Yb + out_row(g, a.divUV, a.divV, m) * g.ldy + ncol, val);
            }
        }
    } else {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int64_t m = m0 + wm * TM + mi * 32 + lrow;
            if (m >= g.M) continue;
            const int64_t orow = out_row(g, a.divUV, a.divV, m);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const f32x16 t = acc_tile(mi, ni);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int nl = wn * TN + ni * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
                    const int ncol = n0 + nl;
                    if (ncol >= g.NC) continue;
                    float v = t[e] * colmul[nl] + coladd[nl];
                    const int64_t off = orow * g.ldy + ncol;
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
    TWN_TRACE_POINT(5);
}

// Sums the split-K partials in a fixed order and applies the block tail:
// y = relu?((0.5*alpha*sum)*scale + shift + residual).  One thread per VEC consecutive output elements.
template <int BM, int BN, int WM, int WN, int STAGES, bool GEMM, bool SPLITK, bool BUF, int OCC = 0>
__global__ __launch_bounds__(64 * WM * WN, OCC ? OCC : dma_min_blocks(WM * WN, STAGES * (BM * 128 + BN * 16)))
void gather_gemm_dma_kernel(const DmaArgs a) {
    gather_gemm_dma_body<BM, BN, WM, WN, STAGES, GEMM, SPLITK, BUF>(a, gridDim.x, blockIdx.x, blockIdx.y);
}

// Up to four problems of the same tile shape in one launch (blockIdx.y = problem): the residue classes of a strided
// backward-data pass, which are too small to be worth a launch each.  The grid is as wide as the largest problem;
// the surplus workgroups of the others leave at once.
constexpr int kDmaBatchMax = 4;
struct DmaBatchArgs {
    DmaArgs p[kDmaBatchMax];
    uint32_t blocks[kDmaBatchMax];
};
template <int BM, int BN, int WM, int WN, int STAGES, bool BUF>
__global__ __launch_bounds__(64 * WM * WN, dma_min_blocks(WM * WN, STAGES * (BM * 128 + BN * 16)))
void gather_gemm_dma_batch_kernel(const DmaBatchArgs ba) {
    const uint32_t c = blockIdx.y;
    const uint32_t nb = ba.blocks[c];
    if (blockIdx.x >= nb) return;           // whole workgroup, before any barrier
    gather_gemm_dma_body<BM, BN, WM, WN, STAGES, false, false, BUF>(ba.p[c], nb, blockIdx.x, 0u);
}

template <int VEC>
__global__ __launch_bounds__(256) void splitk_finish_kernel(const GatherGemm g) {
    const int64_t id0 = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) * VEC;
    const int64_t total = g.M * g.NC;
    if (id0 >= total) return;
    const int64_t m = id0 / g.NC;
    const int ncol0 = static_cast<int>(id0 - m * g.NC);      // VEC = 4 needs NC % 4 == 0: the group stays in one row
    int64_t orow = m;
    if (g.orU != 0) {
        const int64_t uv = static_cast<int64_t>(g.orU) * g.orV;
        const int64_t n = m / uv, rem = m - n * uv;
        const int64_t u = rem / g.orV, v = rem - u * g.orV;
        orow = (n * g.orH + g.ora + g.orsh * u) * g.orW + g.orb + g.orsw * v;
    }
    float s[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) s[v] = 0.0f;
#pragma unroll 8
    for (int sp = 0; sp < g.splits; ++sp) {
        const float* src = g.partial + static_cast<int64_t>(sp) * total + id0;
        if (VEC == 4) {
            const f32x4 t = *reinterpret_cast<const f32x4*>(src);
            s[0] += t[0]; s[1 % VEC] += t[1]; s[2 % VEC] += t[2]; s[3 % VEC] += t[3];
        } else {
            s[0] += src[0];
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const int ncol = ncol0 + e;
        const float mul = 0.5f * g.alpha[ncol / g.rows_per_group] * (g.scale ? g.scale[ncol] : 1.0f);
        float v = s[e] * mul + (g.shift ? g.shift[ncol] : 0.0f);
        const int64_t off = orow * g.ldy + ncol;
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

template <int BM, int BN, int WM, int WN, int STAGES, bool GEMM, bool SPLITK, bool BUF, int OCC>
static int32_t launch_dma_kernel_b(const DmaArgs& a, int64_t blocks, hipStream_t st) {
    constexpr int SMEM = STAGES * (BM * 128 + BN * 16);
    static_assert(SMEM <= 160 * 1024, "LDS budget");
    // more than 64 KB of dynamic LDS has to be allowed once per kernel
    auto k = gather_gemm_dma_kernel<BM, BN, WM, WN, STAGES, GEMM, SPLITK, BUF, OCC>;
    static std::once_flag once;
    static bool allowed = false;
    std::call_once(once, [&] {
        allowed = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      SMEM) == hipSuccess;
    });
    if (!allowed) return TWN_ERR_HIP;
    k<<<dim3(static_cast<unsigned>(blocks), SPLITK ? a.g.splits : 1), dim3(64 * WM * WN), SMEM, st>>>(a);
    return launch_status();
}

template <int BM, int BN, int WM, int WN, int STAGES, bool GEMM, bool SPLITK, int OCC>
static int32_t launch_dma_kernel(const DmaArgs& a, int64_t blocks, hipStream_t st) {
    return a.use_buf ? launch_dma_kernel_b<BM, BN, WM, WN, STAGES, GEMM, SPLITK, true, OCC>(a, blocks, st)
                     : launch_dma_kernel_b<BM, BN, WM, WN, STAGES, GEMM, SPLITK, false, OCC>(a, blocks, st);
}

static DmaArgs make_dma_args(const GatherGemm& g) {
    DmaArgs a;
    a.g = g;
    a.divIC = make_fastdiv_u(static_cast<uint32_t>(g.IC));
    a.divS = make_fastdiv_u(static_cast<uint32_t>(g.S));
    a.divUV = make_fastdiv_u(g.orU ? static_cast<uint32_t>(g.orU) * static_cast<uint32_t>(g.orV) : 1u);
    a.divV = make_fastdiv_u(g.orU ? static_cast<uint32_t>(g.orV) : 1u);
    a.divOW = make_fastdiv_u(static_cast<uint32_t>(g.OW));
    a.divOH = make_fastdiv_u(static_cast<uint32_t>(g.OH));
    {
        // whole-tensor sizes for the buffer descriptors (the last pixel row ends after its IC / K values)
        const int64_t in_rows = g.plain_gemm ? g.M : (g.M / (static_cast<int64_t>(g.OH) * g.OW)) * g.IH * g.IW;
        const int64_t xb = ((in_rows - 1) * g.xs + (g.plain_gemm ? g.K : g.IC)) * 2;
        const int64_t wb = static_cast<int64_t>(g.NC) * g.wpr * 4;
        const bool shape_ok = g.plain_gemm ? (g.K % 64 == 0)
                                           : (g.divh == 1 && g.divw == 1 && g.IC % 64 == 0 && !g.chunk_gather &&
                                              g.M % (static_cast<int64_t>(g.OH) * g.OW) == 0);
        a.use_buf = (env_int("TWN_BUFLOAD", 1) != 0 && shape_ok && xb > 0 && xb < (1LL << 31) && wb < (1LL << 31)) ? 1 : 0;
        a.x_bytes = static_cast<uint32_t>(xb < (1LL << 31) ? xb : 0);
        a.w_bytes = static_cast<uint32_t>(wb < (1LL << 31) ? wb : 0);
    }
    return a;
}

template <int BM, int BN, int WM, int WN, int STAGES, int OCC = 0>
static int32_t launch_dma_tile(const GatherGemm& g, hipStream_t st) {
    const int64_t blocks = ((g.M + BM - 1) / BM) * ((g.NC + BN - 1) / BN);
    if (blocks <= 0 || blocks >= (1LL << 31)) return TWN_ERR_SHAPE;
    const DmaArgs a = make_dma_args(g);
    if (g.splits > 1) {
        // the dispatcher splits K only for grids of few 128x128 tiles: no other tile has a split-K build
        if constexpr (BM == 128 && BN == 128 && WM == 2 && WN == 2) {
            if (!g.partial) return TWN_ERR_WORKSPACE;
            int32_t rc = g.plain_gemm ? launch_dma_kernel<BM, BN, WM, WN, STAGES, true, true, OCC>(a, blocks, st)
                                      : launch_dma_kernel<BM, BN, WM, WN, STAGES, false, true, OCC>(a, blocks, st);
            if (rc != TWN_OK) return rc;
            const int64_t total = g.M * g.NC;
            if (g.NC % 4 == 0 && (reinterpret_cast<uintptr_t>(g.partial) & 15) == 0)
                splitk_finish_kernel<4><<<static_cast<unsigned>((total / 4 + 255) / 256), 256, 0, st>>>(g);
            else
                splitk_finish_kernel<1><<<static_cast<unsigned>((total + 255) / 256), 256, 0, st>>>(g);
            return launch_status();
        } else {
            return TWN_ERR_UNSUPPORTED;
        }
    }
    return g.plain_gemm ? launch_dma_kernel<BM, BN, WM, WN, STAGES, true, false, OCC>(a, blocks, st)
                        : launch_dma_kernel<BM, BN, WM, WN, STAGES, false, false, OCC>(a, blocks, st);
}

// Tile ids (BM x BN, waves, stages): 12 = 128x128 2x2 S3, 14 = 64x128 1x4 S3, 15 = 128x128 1x4 S3,
// 16 = 128x64 2x2 S3,
// 17 = 128x256 1x4 S4, 24 = 128x512 1x8 S4, 30 = 256x256 2x2 S3
// (30: 16 accumulator tiles per wave, pinned by hand; only on request, it is not faster than 17)
#ifdef TWN_TRACE
extern "C" int32_t twn_debug_set_trace(void* buf) {
    uint64_t* p = static_cast<uint64_t*>(buf);
    return hipMemcpyToSymbol(HIP_SYMBOL(g_trace), &p, sizeof(p)) == hipSuccess ? 0 : -6;
}
#endif

template <int BM, int BN, int WM, int WN, int STAGES, bool BUF>
static int32_t launch_dma_batch_kernel(const DmaBatchArgs& ba, unsigned width, int count, hipStream_t st) {
    constexpr int SMEM = STAGES * (BM * 128 + BN * 16);
    auto k = gather_gemm_dma_batch_kernel<BM, BN, WM, WN, STAGES, BUF>;
    static std::once_flag once;
    static bool allowed = false;
    std::call_once(once, [&] {
        allowed = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      SMEM) == hipSuccess;
    });
    if (!allowed) return TWN_ERR_HIP;
    k<<<dim3(width, static_cast<unsigned>(count)), dim3(64 * WM * WN), SMEM, st>>>(ba);
    return launch_status();
}

template <int BM, int BN, int WM, int WN, int STAGES>
static int32_t launch_dma_batch_tile(const GatherGemm* gs, int count, hipStream_t st) {
    DmaBatchArgs ba{};
    int64_t width = 0;
    bool buf = true;
    for (int c = 0; c < count; ++c) {
        const GatherGemm& g = gs[c];
        if (g.splits > 1 || g.plain_gemm) return TWN_ERR_UNSUPPORTED;
        const int64_t blocks = ((g.M + BM - 1) / BM) * ((g.NC + BN - 1) / BN);
        if (blocks <= 0 || blocks >= (1LL << 31)) return TWN_ERR_SHAPE;
        ba.p[c] = make_dma_args(g);
        ba.blocks[c] = static_cast<uint32_t>(blocks);
        if (blocks > width) width = blocks;
        buf = buf && ba.p[c].use_buf;
    }
    // one build serves all problems of the launch: buffer-descriptor loads only if every problem qualifies
    return buf ? launch_dma_batch_kernel<BM, BN, WM, WN, STAGES, true>(ba, static_cast<unsigned>(width), count, st)
               : launch_dma_batch_kernel<BM, BN, WM, WN, STAGES, false>(ba, static_cast<unsigned>(width), count, st);
}

// `count` <= 4 unsplit convolution problems with the same tile id in one launch.
int32_t launch_gather_gemm_dma_batch(const GatherGemm* gs, int count, int tile, hipStream_t st) {
    if (count < 1 || count > kDmaBatchMax) return TWN_ERR_UNSUPPORTED;
    switch (tile) {
        case 12: return launch_dma_batch_tile<128, 128, 2, 2, 3>(gs, count, st);
        case 14: return launch_dma_batch_tile<64, 128, 1, 4, 3>(gs, count, st);
        case 15: return launch_dma_batch_tile<128, 128, 1, 4, 3>(gs, count, st);
        case 16: return launch_dma_batch_tile<128, 64, 2, 2, 3>(gs, count, st);
        default: return TWN_ERR_UNSUPPORTED;
    }
}

int32_t launch_gather_gemm_dma(const GatherGemm& g, int tile, hipStream_t st) {
    switch (tile) {
        case 12: return launch_dma_tile<128, 128, 2, 2, 3>(g, st);
        case 14: return launch_dma_tile<64, 128, 1, 4, 3>(g, st);
        case 15: return launch_dma_tile<128, 128, 1, 4, 3>(g, st);
        case 16: return launch_dma_tile<128, 64, 2, 2, 3>(g, st);
        case 17: return launch_dma_tile<128, 256, 1, 4, 4>(g, st);
        case 24: return launch_dma_tile<128, 512, 1, 8, 4>(g, st);
        case 30: return launch_dma_tile<256, 256, 2, 2, 3>(g, st);
        default: return TWN_ERR_UNSUPPORTED;
    }
}

}  // namespace twn
