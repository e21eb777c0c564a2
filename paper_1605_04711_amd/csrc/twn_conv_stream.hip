// Persistent implicit-GEMM ternary convolution / inner product on gfx950
// (Eq. 2, Alg. 1 step 8; also the undivided backward-data pass of Alg. 1 step 9).
//
// Same arithmetic and the same per-slab pipeline as gather_gemm_dma_kernel (bf16
// activations staged global -> LDS by direct 16-byte buffer loads, 2-bit codes
// expanded in registers to +-2.0 / 0, v_mfma_f32_32x32x16_bf16, alpha/2 in the fp32
// epilogue), but a workgroup does not end with its tile.  The grid is sized to what
// the chip holds at once and every workgroup walks a list of tiles; the K slabs of
// all its tiles form ONE stream:
//   * the loads of the next tile's first slabs are issued while the last slabs of the
//     current tile are multiplied, so no tile after the first waits for memory at its
//     start and nothing is drained at its end;
//   * the epilogue of a tile (scale, shift, residual, ReLU, rounding, transposition
//     through LDS, 16-byte stores) runs while those loads are in flight; it stages
//     through the one pipeline stage that is free at that moment (the stage of the
//     slab just multiplied; the next load to it is issued only after the following
//     mid-slab barrier), 32 pixel rows per wave at a time;
//   * co-resident workgroups drift out of step, so the vector-ALU work of one
//     workgroup's epilogue and tile set-up overlaps the MFMAs of the others instead
//     of every workgroup of a launch doing the same phase at the same time;
//   * per-column parameters (alpha, scale, shift) are loaded one tile ahead.
// Shapes it takes: bf16 output, channel counts that are multiples of 8, and the
// loads of the buffer-descriptor path (plain GEMM with K % 64 == 0, or an undivided
// convolution whose channel count is a multiple of 64; tensors below 2 GiB).  Every
// other problem stays with gather_gemm_dma_kernel.
#include <mutex>

#include "twn_kernels.h"
#include "twn_lds_asm.h"
#include "twn_mfma.h"
#include "twn_stream_epilogue.h"

namespace twn {

#ifdef TWN_TRACE
// development build only: per-workgroup phase timestamps (shader clock), 16 slots per workgroup
__device__ uint64_t* g_stream_trace = nullptr;
#define TWN_STRACE(slot)                                                                                   \
    do {                                                                                                   \
        if (g_stream_trace && threadIdx.x == 0 && (slot) < 16)                                             \
            g_stream_trace[static_cast<size_t>(blockIdx.x) * 16 + (slot)] = __builtin_readcyclecounter();  \
    } while (0)
extern "C" int32_t twn_debug_set_stream_trace(void* buf) {
    uint64_t* p = static_cast<uint64_t*>(buf);
    return hipMemcpyToSymbol(HIP_SYMBOL(g_stream_trace), &p, sizeof(p)) == hipSuccess ? 0 : -6;
}
#else
#define TWN_STRACE(slot) do {} while (0)
#endif

struct StreamArgs {
    GatherGemm g;
    FastDivU divOW, divOH;      // GEMM row -> (image, oh, ow)
    FastDivU divTN;             // tile -> (row block, column block)
    uint32_t x_bytes, w_bytes, y_bytes;  // sizes for the buffer descriptors
    uint32_t tiles, tiles_n;
    int32_t KT;                 // K / 64
};

template <int BM, int BN, int WM, int WN, int STAGES, bool GEMM, int OCC, int KS>
// (the second launch bound is in waves per SIMD)
__global__ __launch_bounds__(64 * WM * WN * KS, (OCC * WM * WN * KS + 3) / 4)
void conv_stream_kernel(const StreamArgs a) {
    // KS > 1: the workgroup holds KS groups of WM*WN waves.  All groups work on the SAME output tile; group kg
    // takes the K slabs kg, kg+KS, kg+2KS, ... (it stages and multiplies them on its own, in its own part of
    // every stage), and the partial tiles are summed through LDS in a fixed order before the epilogue.  This
    // multiplies the waves per CU for layers with too few tiles to fill the chip (few pixels, deep K).
    constexpr int NWG = WM * WN;                   // waves per K group
    constexpr int NW = NWG * KS;                   // waves per workgroup
    constexpr int NT = 64 * NW;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int NLOAD = BM / (8 * NWG);          // 1 KB (8 rows) per wave-level load
    constexpr int A_BYTES = BM * 128;
    constexpr int B_BYTES = BN * 16;
    constexpr int SUB_BYTES = A_BYTES + B_BYTES;   // one slab of one K group
    constexpr int STAGE_BYTES = KS * SUB_BYTES;
    constexpr int PD = STAGES - 1;                 // slabs in flight ahead of the one being multiplied
    constexpr int PER_STAGE = NLOAD + 1;           // vector-memory loads per wave per slab
    constexpr int EPI_CH = TN < 64 ? TN : 64;      // channels staged at a time
    constexpr int EPI_ROW = EPI_CH * 2 + 16;       // bytes per staged pixel row (pad keeps 16-byte reads conflict-free)
    constexpr int EPI_WAVE = 32 * EPI_ROW;         // one block of 32 pixel rows per wave
    static_assert(BM % (8 * NWG) == 0 && BN % 64 == 0 && BN <= 64 * NWG && TN % 32 == 0 && TM % 32 == 0, "tile shape");
    static_assert(NWG % 2 == 0, "the swizzle of the staged rows assumes an even number of waves");
    static_assert(STAGES >= 3, "the mid-slab hand-over needs two slabs in flight");
    static_assert(NWG * EPI_WAVE <= STAGE_BYTES, "epilogue staging must fit in one pipeline stage");
    static_assert(KS == 1 || KS == 2 || KS == 4, "K groups");
    // partial tiles of a K group pass through the free stage RED_MI row blocks (of 32 pixels) at a time
    constexpr int RED_MI_FIT = STAGE_BYTES / (NWG * NI * 4096);
    constexpr int RED_MI = RED_MI_FIT < MI ? RED_MI_FIT : MI;
    static_assert(KS == 1 || (RED_MI >= 1 && MI % RED_MI == 0), "the reduction must fit in the free stage");
    // Column parameters of a tile: a region of their own behind the stages (double-buffered, no extra barrier),
    // unless that region would cost a resident workgroup; then they share the free stage with the staging
    // rows, at the price of a second barrier per tile.
    constexpr bool COL_IN_STAGE = (STAGES * STAGE_BYTES + 4 * BN * 4) * OCC > 160 * 1024;
    static_assert(!COL_IN_STAGE || NWG * EPI_WAVE + 2 * BN * 4 <= STAGE_BYTES, "column parameters must fit in the free stage");
    static_assert(BN <= NT, "one thread per column loads the column parameters");
    static_assert(MI <= 8 && NI <= 4, "fragment reads use immediate offsets");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    float* colbuf = reinterpret_cast<float*>(smem + STAGES * STAGE_BYTES);   // [2][2][BN]: mul, add of even / odd tiles (unless COL_IN_STAGE)

    TWN_STRACE(0);
#ifdef TWN_TRACE
    if (g_stream_trace && threadIdx.x == 0) g_stream_trace[static_cast<size_t>(blockIdx.x) * 16 + 15] = wall_clock64();
#endif
    const GatherGemm& g = a.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = wave / NWG, wv = wave % NWG;    // K group, wave inside the group
    const int wm = wv / WN, wn = wv % WN;
    const int lrow = lane & 31, lh = lane >> 5;

    // ---- this workgroup's tiles ------------------------------------------------------------------
    // Workgroups are dealt round-robin to the 8 XCDs.  Each XCD owns a contiguous range of tiles and its
    // workgroups walk that range side by side: the tiles in flight on one XCD are neighbours (shared halos
    // and codes in its L2).
    const uint32_t G = gridDim.x, b = blockIdx.x;
    const uint32_t xcd = b & 7, j = b >> 3;
    const uint32_t gx = (G + 7 - xcd) >> 3;                 // workgroups on this XCD
    const uint32_t q = a.tiles >> 3, r = a.tiles & 7;
    const uint32_t count_x = q + (xcd < r ? 1u : 0u);       // tiles of this XCD
    const uint32_t start_x = xcd * q + (xcd < r ? xcd : r);
    if (j >= count_x) return;                               // whole workgroup, before any barrier
    const uint32_t n_my = (count_x - j + gx - 1) / gx;
    auto tile_id = [&](uint32_t i) __attribute__((always_inline)) -> uint32_t { return start_x + j + i * gx; };

    const int KT = a.KT;                           // 64-wide slabs of K
    const int KTS = (KT + KS - 1) / KS;            // slabs per K group (the last one of a group may be empty)
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(g.X, a.x_bytes), rw = make_rsrc(g.Wq, a.w_bytes);

    // ---- per-lane load state of the tile the load stream is in ----------------------------------------
    // wave-level load i covers rows (i*NWG + wv)*8 .. +7 of the tile; LDS row r keeps logical 16-byte chunk
    // c at position c ^ ((r >> 1) & 7) (conflict-free ds_read_b128 with 64 banks); the swizzle is applied by
    // choosing which chunk of the row this lane fetches.
    const int kc = (lane & 7) ^ ((wv & 1) * 4 + ((lane >> 4) & 3));
    const int brow = (wv * 64) % BN + lane;                 // column whose codes this lane stages
    uint32_t voffA[NLOAD];      // GEMM: byte offset of the row; convolution: byte offset of tap (0,0) (any sign, wraps)
    int ih0[NLOAD], iw0[NLOAD];
    uint32_t voffB;
    auto tile_setup = [&](uint32_t t, bool valid) __attribute__((always_inline)) {
        const uint32_t tm = fdiv_u(t, a.divTN);
        const uint32_t tn = t - tm * a.tiles_n;
        const uint32_t m0 = tm * BM;
        const uint32_t ncol = tn * BN + static_cast<uint32_t>(brow);
        voffB = (valid && ncol < static_cast<uint32_t>(g.NC)) ? ncol * static_cast<uint32_t>(g.wpr) * 4u : kBufOutside;
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            const uint32_t m = m0 + static_cast<uint32_t>((i * NWG + wv) * 8 + (lane >> 3));
            // computed unconditionally and selected afterwards (no memory is touched here)
            const bool rv = valid && m < static_cast<uint32_t>(g.M);
            uint32_t vo;
            int h0 = 0, w0 = 0;
            if (GEMM) {
                vo = (m * static_cast<uint32_t>(g.xs) + static_cast<uint32_t>(kc * 8)) * 2u;
            } else {
                const uint32_t tt = fdiv_u(m, a.divOW);
                const int ow = static_cast<int>(m - tt * static_cast<uint32_t>(g.OW));
                const uint32_t img = fdiv_u(tt, a.divOH);
                const int oh = static_cast<int>(tt - img * static_cast<uint32_t>(g.OH));
                h0 = oh * g.sh - g.ph;
                w0 = ow * g.sw - g.pw;
                // 32-bit wrapping arithmetic: the true offset of every tap that passes the bounds test
                // lies in [0, 2^31)
                const uint32_t pix = (img * static_cast<uint32_t>(g.IH) + static_cast<uint32_t>(h0)) *
                                         static_cast<uint32_t>(g.IW) + static_cast<uint32_t>(w0);
                vo = (pix * static_cast<uint32_t>(g.xs) + static_cast<uint32_t>(kc * 8)) * 2u;
            }
            voffA[i] = rv ? vo : kBufOutside;
            ih0[i] = rv ? h0 : -(1 << 28);
            iw0[i] = rv ? w0 : -(1 << 28);
        }
    };

    // ---- the load stream: (tile lt, slab lk), wave-uniform ----------------------------------------------
    uint32_t lt = 0;
    int lk = 0;                         // slab of this K group inside the tile: K slab lk*KS + kg
    int nc0 = 0, nss = 0, nrr = 0;      // convolution: channel base and tap of the slab to issue next
    // carries of the (channel base, tap column, tap row) counter; at most KS of them per advance
    auto tap_normalize = [&]() __attribute__((always_inline)) {
        while (nc0 >= g.IC) {
            nc0 -= g.IC;
            if (++nss == g.S) {
                nss = 0;
                ++nrr;
            }
        }
    };
    auto tap_reset = [&]() __attribute__((always_inline)) {
        nc0 = 64 * kg;
        nss = nrr = 0;
        if (KS > 1) tap_normalize();
    };
    const int32_t strR = g.dh * g.IW * static_cast<int>(g.xs) * 2, strS = g.dw * static_cast<int>(g.xs) * 2;
    struct {
        unsigned char* sbase;
        bool in_k;                      // KS > 1: false for the empty last slab of a group (every lane reads zeros)
        uint32_t soff;                  // slab index inside the tile
        int32_t delta_b;                // convolution: byte offset of this slab's tap and channel base
        int dth, dtw;
    } si;
    auto issue_setup = [&](int stage) __attribute__((always_inline)) {
        si.sbase = smem + stage * STAGE_BYTES + kg * SUB_BYTES;
        si.soff = static_cast<uint32_t>(lk * KS + kg);
        si.in_k = (KS == 1) || (lk * KS + kg < KT);
        if (!GEMM) {
            si.delta_b = nrr * strR + nss * strS + nc0 * 2;
            si.dth = nrr * g.dh;
            si.dtw = nss * g.dw;
        }
    };
    auto issue_load = [&](auto i_tag) __attribute__((always_inline)) {
        constexpr int i = decltype(i_tag)::value;
        if constexpr (i == NLOAD) {
            buf_dma16(rw, si.in_k ? voffB : kBufOutside, si.soff * 16u, si.sbase + A_BYTES + ((wv * 64) % BN) * 16);
        } else if (GEMM) {
            buf_dma16(rx, si.in_k ? voffA[i] : kBufOutside, si.soff * 128u, si.sbase + (i * NWG + wv) * 1024);
        } else {
            const bool ok = (static_cast<unsigned>(ih0[i] + si.dth) < static_cast<unsigned>(g.IH)) &
                            (static_cast<unsigned>(iw0[i] + si.dtw) < static_cast<unsigned>(g.IW)) & si.in_k;
            buf_dma16(rx, ok ? voffA[i] + static_cast<uint32_t>(si.delta_b) : kBufOutside, 0u,
                      si.sbase + (i * NWG + wv) * 1024);
        }
    };
    // after the last load of a slab: next slab, or the first slab of the next tile (past the last tile every
    // lane reads zeros: the loads keep their count, which the vmcnt arithmetic below relies on)
    auto issue_advance = [&]() __attribute__((always_inline)) {
        ++lk;
        if (!GEMM) {
            nc0 += 64 * KS;
            tap_normalize();
        }
        if (lk == KTS) {
            lk = 0;
            if (!GEMM) tap_reset();
            ++lt;
            tile_setup(tile_id(lt), lt < n_my);
        }
    };

    // ---- per-column parameters, loaded one tile ahead (thread c < BN owns column c of the tile) --------
    float cp_alpha = 0.0f, cp_scale = 1.0f, cp_shift = 0.0f;
    auto colparam_load = [&](uint32_t t) __attribute__((always_inline)) {
        const uint32_t tm = fdiv_u(t, a.divTN);
        const int ncol = static_cast<int>((t - tm * a.tiles_n) * BN) + tid;
        cp_alpha = 0.0f;
        cp_scale = 1.0f;
        cp_shift = 0.0f;
        if (tid < BN && ncol < g.NC) {
            const int ag = (g.rows_per_group >= g.NC) ? 0 : ncol / g.rows_per_group;
            cp_alpha = g.alpha[ag];
            if (g.scale) cp_scale = g.scale[ncol];
            if (g.shift) cp_shift = g.shift[ncol];
        }
    };

    f32x16 acc[MI][NI];
    auto acc_clear = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.0f;
    };

    // ---- software pipeline (see gather_gemm_dma_kernel for the reasoning behind its shape) --------------
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) unsigned char*)smem));
    uint32_t aoff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        aoff[kk] = kg * SUB_BYTES + (wm * TM + lrow) * 128 + (((lh * 4 + kk) ^ ((lrow >> 1) & 7)) * 16);
    const uint32_t boff = kg * SUB_BYTES + A_BYTES + (wn * TN + lrow) * 16 + lh * 8;

    u32x2 breg[2][NI];      // packed codes of the slab being multiplied / of the next slab
    u32x4 afrag[2][MI];     // activation fragments of step kk in set kk & 1
    u32x4 bfrag[2][NI];     // expanded codes of step kk in set kk & 1

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

    auto step = [&](auto kk_tag, auto cur_tag, int stage, int next, int fill) __attribute__((always_inline)) {
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
                constexpr int qq = p - P_RA - P_RB;
                expand(std::integral_constant<int, KN>{}, std::integral_constant<int, qq / 4>{},
                       std::integral_constant<int, qq % 4>{}, breg[BSRC], bfrag[NSET]);
            } else {
                constexpr int gi = G0 + p - (P_RA + P_RB + P_D);
                if constexpr (gi == 0) issue_setup(fill);
                issue_load(std::integral_constant<int, gi>{});
                if constexpr (gi == NLOAD) issue_advance();
            }
        };
        static_for<NM>([&](auto j_tag) __attribute__((always_inline)) {
            constexpr int jj = decltype(j_tag)::value;
            constexpr int mi = jj / NI, ni = jj % NI;
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfrag[SET][ni]),
                                                                  __builtin_bit_cast(bf16x8, afrag[SET][mi]),
                                                                  acc[mi][ni], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            static_for<P>([&](auto p_tag) __attribute__((always_inline)) {
                constexpr int p = decltype(p_tag)::value;
                if constexpr (p * NM / P == jj) piece(p_tag);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        lds_wait<0>();
        lds_ready<MI>(afrag[NSET]);
        if constexpr (KK == 2) lds_ready<NI>(breg[CUR ^ 1]);
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- epilogue of the tile the compute stream has just finished -------------------------------------
    const uint32_t ldyB = static_cast<uint32_t>(g.ldy) * 2u;
    TileStoreLane<EPI_CH> store_lane;
    store_lane.init(lane, ldyB);
    uint32_t ct = 0;        // tiles finished so far
    auto epilogue = [&](int free_stage) __attribute__((always_inline)) {
        float* cmul = colbuf + (ct & 1u) * (2 * BN);
        if constexpr (COL_IN_STAGE) {
            // the free stage may still be read by slower waves
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            cmul = reinterpret_cast<float*>(smem + free_stage * STAGE_BYTES + NWG * EPI_WAVE);
        }
        float* cadd = cmul + BN;
        if (tid < BN) {
            cmul[tid] = 0.5f * cp_alpha * cp_scale;      // codes were +-2
            cadd[tid] = cp_shift;
        }
        // every wave has finished reading the stage of the last slab, and the column parameters are visible:
        // a bare s_barrier does not wait for this wave's LDS writes, so they are waited for first
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if constexpr (KS > 1) {
            // Sum of the K groups' partial tiles, in a fixed order (group 1, then 2, ...), through the free
            // stage: a lane of group kg writes the accumulator quads of RED_MI row blocks, the same lane of
            // group 0 adds them.  Every wave takes part in every barrier.
            f32x4* red = reinterpret_cast<f32x4*>(smem + free_stage * STAGE_BYTES);
#pragma unroll
            for (int src = 1; src < KS; ++src) {
#pragma unroll
                for (int c0 = 0; c0 < MI; c0 += RED_MI) {
                    if (kg == src) {
#pragma unroll
                        for (int mi = 0; mi < RED_MI; ++mi)
#pragma unroll
                            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                                for (int q4 = 0; q4 < 4; ++q4) {
                                    const f32x16& t = acc[c0 + mi][ni];
                                    red[(((wv * RED_MI + mi) * NI + ni) * 4 + q4) * 64 + lane] =
                                        f32x4{t[q4 * 4], t[q4 * 4 + 1], t[q4 * 4 + 2], t[q4 * 4 + 3]};
                                }
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                    if (kg == 0) {
#pragma unroll
                        for (int mi = 0; mi < RED_MI; ++mi)
#pragma unroll
                            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                                for (int q4 = 0; q4 < 4; ++q4) {
                                    const f32x4 v = red[(((wv * RED_MI + mi) * NI + ni) * 4 + q4) * 64 + lane];
#pragma unroll
                                    for (int e = 0; e < 4; ++e) acc[c0 + mi][ni][q4 * 4 + e] += v[e];
                                }
                    }
                    // the sums are in registers (their LDS reads have returned) before the region is reused
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
            }
        }
        const uint32_t t = tile_id(ct);
        const uint32_t tm = fdiv_u(t, a.divTN);
        const uint32_t m0 = tm * BM;
        const int n0 = static_cast<int>((t - tm * a.tiles_n) * BN);
        // the output descriptors are built here, per tile: scalar registers are scarce in the main loop
        uint32_t yb = a.y_bytes;
        asm volatile("" : "+s"(yb));
        const __amdgpu_buffer_rsrc_t ry = make_rsrc(g.Y, yb);
        const __amdgpu_buffer_rsrc_t rr = make_rsrc(g.residual ? g.residual : g.Y, yb);
        const uint32_t relu_floor = g.relu ? 0u : 0x80008000u;
        if (KS == 1 || kg == 0)
            store_tile_bf16<MI, NI, EPI_CH>(acc, cmul + wn * TN, cadd + wn * TN, smem + free_stage * STAGE_BYTES + wv * EPI_WAVE,
                                            store_lane, ry, rr, g.residual != nullptr, m0 + static_cast<uint32_t>(wm * TM),
                                            n0 + wn * TN, static_cast<uint32_t>(g.M), g.NC, ldyB, relu_floor, lane);
        acc_clear();
        ++ct;
        if (ct < n_my) colparam_load(tile_id(ct));
    };

    // ---- prologue: column parameters of the first tile, PD slabs in flight, the first one landed ------------
    colparam_load(tile_id(0));
    if (!GEMM) tap_reset();
    tile_setup(tile_id(0), true);
#pragma unroll
    for (int s = 0; s < PD; ++s) {
        issue_setup(s % STAGES);
        static_for<NLOAD + 1>(issue_load);
        issue_advance();
    }
    acc_clear();
    TWN_STRACE(1);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm((PD - 1) * PER_STAGE));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    TWN_STRACE(2);
    lds_read64_n<NI, 32 * 16>(breg[0], lds_base + boff);
    lds_read128_n<MI, 32 * 128>(afrag[0], lds_base + aoff[0]);
    lds_wait<0>();
    lds_ready<NI>(breg[0]);
    lds_ready<MI>(afrag[0]);
    static_for<4 * NI>([&](auto q_tag) __attribute__((always_inline)) {
        constexpr int qq = decltype(q_tag)::value;
        expand(std::integral_constant<int, 0>{}, std::integral_constant<int, qq / 4>{},
               std::integral_constant<int, qq % 4>{}, breg[0], bfrag[0]);
    });

    int stage = 0;          // stage of the slab being multiplied
    int fill = PD % STAGES; // stage that the slab PD positions ahead goes to
    int kt = 0;             // slab of the current tile
    // one slab of the stream; CUR selects the register set holding this slab's packed codes
    auto slab = [&](auto cur_tag) __attribute__((always_inline)) {
        const int next = (stage + 1 == STAGES) ? 0 : stage + 1;
        {
#ifdef TWN_TRACE
            // fine-grained timeline of one slab (every step ends with lgkmcnt(0), which also covers s_memtime)
            uint64_t ts[7];
#define TWN_TS(i) asm volatile("s_memtime %0" : "=s"(ts[i]))
#else
#define TWN_TS(i) do {} while (0)
#endif
            TWN_TS(0);
            step(std::integral_constant<int, 0>{}, cur_tag, stage, next, fill);
            TWN_TS(1);
            step(std::integral_constant<int, 1>{}, cur_tag, stage, next, fill);
            // hand-over: the next slab of the stream has landed (the PD-2 younger slabs may stay in flight), the
            // stage of the previous slab is free
            TWN_TS(2);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(vmcnt_imm((PD - 2) * PER_STAGE));
            TWN_TS(3);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            TWN_TS(4);
            step(std::integral_constant<int, 2>{}, cur_tag, stage, next, fill);
            TWN_TS(5);
            step(std::integral_constant<int, 3>{}, cur_tag, stage, next, fill);
            TWN_TS(6);
#ifdef TWN_TRACE
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (g_stream_trace && threadIdx.x == 0 && ct == 0 && kt == 5) {
                for (int i = 0; i < 7; ++i) g_stream_trace[static_cast<size_t>(blockIdx.x) * 16 + 8 + i] = ts[i];
            }
#endif
            const int done = stage;
            stage = next;
            fill = (fill + 1 == STAGES) ? 0 : fill + 1;
            if (++kt == KTS) {
                kt = 0;
                TWN_STRACE(3 + 2 * ct);
                epilogue(done);
                TWN_STRACE(2 + 2 * ct);      // ct was advanced by the epilogue
            }
        }
    };
    const uint32_t total = n_my * static_cast<uint32_t>(KTS);
    for (uint32_t s = 0; s < total; s += 2) {
        slab(std::integral_constant<int, 0>{});
        if (s + 1 < total) slab(std::integral_constant<int, 1>{});
    }
    // the trailing zero loads still target this workgroup's LDS: they must have landed before it ends
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
}

// ---- host side ------------------------------------------------------------------------------------------

bool conv_stream_applicable(const GatherGemm& g) {
    if (g.y_f32 || g.NC % 8 != 0 || g.ldy % 8 != 0 || g.orU != 0 || g.splits > 1 || g.chunk_gather) return false;
    if (g.M <= 0 || g.M >= (1LL << 31) - 1024) return false;
    if (g.plain_gemm) {
        if (g.K % 64 != 0 || g.xs % 8 != 0) return false;
    } else {
        if (g.divh != 1 || g.divw != 1 || g.IC % 64 != 0 || g.xs % 8 != 0) return false;
        if (g.M % (static_cast<int64_t>(g.OH) * g.OW) != 0) return false;
    }
    if (!aligned(g.X, 16) || !aligned(g.Wq, 16) || !aligned(g.Y, 16) || (g.residual && !aligned(g.residual, 8))) return false;
    const int64_t in_rows = g.plain_gemm ? g.M : (g.M / (static_cast<int64_t>(g.OH) * g.OW)) * g.IH * g.IW;
    const int64_t xb = ((in_rows - 1) * g.xs + (g.plain_gemm ? g.K : g.IC)) * 2;
    const int64_t wb = static_cast<int64_t>(g.NC) * g.wpr * 4;
    const int64_t yb = ((g.M - 1) * g.ldy + g.NC) * 2;       // the output path addresses Y and the residual by 32-bit offsets
    return xb > 0 && xb < (1LL << 31) && wb < (1LL << 31) && yb < (1LL << 31);
}

namespace {

int num_cus(hipStream_t) {
    static std::once_flag once;
    static int cus = 256;
    std::call_once(once, [] {
        int dev = 0;
        hipDeviceProp_t p;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess && p.multiProcessorCount > 0)
            cus = p.multiProcessorCount;
    });
    return cus;
}

template <int BM, int BN, int WM, int WN, int STAGES, bool GEMM, int OCC, int KS>
int32_t launch_stream_kernel(const StreamArgs& a, hipStream_t st) {
    constexpr int PIPE = STAGES * KS * (BM * 128 + BN * 16);
    constexpr int SMEM = ((PIPE + 4 * BN * 4) * OCC > 160 * 1024) ? PIPE : PIPE + 4 * BN * 4;   // see COL_IN_STAGE
    static_assert(SMEM <= 160 * 1024, "LDS budget");
    auto k = conv_stream_kernel<BM, BN, WM, WN, STAGES, GEMM, OCC, KS>;
    // more than 64 KB of dynamic LDS has to be allowed once per kernel; the occupancy query sizes the grid
    static std::once_flag once;
    static int per_cu = 0;
    std::call_once(once, [&] {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, SMEM) !=
            hipSuccess)
            return;
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k, 64 * WM * WN * KS, SMEM) == hipSuccess && n > 0) per_cu = n;
    });
    if (per_cu <= 0) return TWN_ERR_HIP;
    int occ = per_cu;
    const int cap = env_int("TWN_STREAM_OCC", 0);
    if (cap > 0 && cap < occ) occ = cap;
    int64_t grid = static_cast<int64_t>(num_cus(st)) * occ;
    if (grid > a.tiles) grid = a.tiles;
    k<<<dim3(static_cast<unsigned>(grid)), dim3(64 * WM * WN * KS), SMEM, st>>>(a);
    return launch_status();
}

template <int BM, int BN, int WM, int WN, int STAGES, int OCC, int KS>
int32_t launch_stream_tile(const GatherGemm& g, hipStream_t st) {
    const int64_t tiles_n = (g.NC + BN - 1) / BN;
    const int64_t tiles = ((g.M + BM - 1) / BM) * tiles_n;
    if (tiles <= 0 || tiles >= (1LL << 31)) return TWN_ERR_SHAPE;
    StreamArgs a;
    a.g = g;
    a.divOW = make_fastdiv_u(static_cast<uint32_t>(g.OW));
    a.divOH = make_fastdiv_u(static_cast<uint32_t>(g.OH));
    a.divTN = make_fastdiv_u(static_cast<uint32_t>(tiles_n));
    const int64_t in_rows = g.plain_gemm ? g.M : (g.M / (static_cast<int64_t>(g.OH) * g.OW)) * g.IH * g.IW;
    a.x_bytes = static_cast<uint32_t>(((in_rows - 1) * g.xs + (g.plain_gemm ? g.K : g.IC)) * 2);
    a.w_bytes = static_cast<uint32_t>(static_cast<int64_t>(g.NC) * g.wpr * 4);
    a.y_bytes = static_cast<uint32_t>(((g.M - 1) * g.ldy + g.NC) * 2);
    a.tiles = static_cast<uint32_t>(tiles);
    a.tiles_n = static_cast<uint32_t>(tiles_n);
    a.KT = g.K / 64;
    return g.plain_gemm ? launch_stream_kernel<BM, BN, WM, WN, STAGES, true, OCC, KS>(a, st)
                        : launch_stream_kernel<BM, BN, WM, WN, STAGES, false, OCC, KS>(a, st);
}

}  // namespace

// Tile ids as in launch_gather_gemm_dma: 12 = 128x128 2x2, 14 = 64x128 1x4, 15 = 128x128 1x4, 16 = 128x64 2x2,
// 17 = 128x256 1x4 (4 stages).  The caller has checked conv_stream_applicable.
int32_t launch_conv_stream(const GatherGemm& g, int tile, hipStream_t st) {
    // K groups: layers whose 64x128 tiles do not even give every CU one workgroup (few pixels, deep K) run two
    // groups of four waves per tile (ResNet-18 stage 4: 31 -> 24 us); TWN_STREAM_KS overrides for experiments
    int ks = env_int("TWN_STREAM_KS", 0);
    // Load waves (conv_stream_pc_kernel): four of them next to the four compute waves.  They pay off where a
    // workgroup has few tiles and a deep K (ResNet-18 stages 3 and 4: 22 -> 19.5 us and 24 -> 20.7 us per 3x3
    // layer), and replace the K groups there; with 128x256 tiles one workgroup of 4 + 4 waves per CU does what two
    // workgroups of four waves did (VGG-16 conv5-7: 5-8 % faster); 128x64 tiles (64 output channels) gain nothing.
    // TWN_STREAM_PC: 0 = never, 2 / 4 = that many load waves wherever a build exists, unset = this rule.
    int np = env_int("TWN_STREAM_PC", -1);
    if (np < 0) np = (tile == 14 || tile == 15 || tile == 17) ? 4 : 0;
    if (np > 0) {
        const int32_t rc = launch_conv_stream_pc(g, tile, ks == 0 ? 1 : ks, np, env_int("TWN_STREAM_PC_STAGES", 4), st);
        if (rc != TWN_ERR_UNSUPPORTED) return rc;
    }
    if (ks == 0) {
        const int64_t tiles64 = ((g.M + 63) / 64) * ((g.NC + 127) / 128);
        ks = (tile == 14 && tiles64 <= 320 && g.K >= 1024) ? 2 : 1;
    }
    switch (tile) {
        case 12: return launch_stream_tile<128, 128, 2, 2, 3, 2, 1>(g, st);
        case 14:
            if (ks == 2) return launch_stream_tile<64, 128, 1, 4, 3, 2, 2>(g, st);
            if (ks == 4) return launch_stream_tile<64, 128, 1, 4, 3, 1, 4>(g, st);
            return launch_stream_tile<64, 128, 1, 4, 3, 4, 1>(g, st);
        case 15:
            if (ks == 2) return launch_stream_tile<128, 128, 1, 4, 3, 1, 2>(g, st);
            return launch_stream_tile<128, 128, 1, 4, 3, 2, 1>(g, st);
        case 16:
            if (ks == 2) return launch_stream_tile<128, 64, 2, 2, 3, 1, 2>(g, st);
            return launch_stream_tile<128, 64, 2, 2, 3, 3, 1>(g, st);
        case 17: return launch_stream_tile<128, 256, 1, 4, 4, 2, 1>(g, st);
        default: return TWN_ERR_UNSUPPORTED;
    }
}

}  // namespace twn
