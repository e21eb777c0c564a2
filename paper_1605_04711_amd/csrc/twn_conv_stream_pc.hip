// Persistent implicit-GEMM ternary convolution / inner product with dedicated load waves, gfx950
// (Eq. 2, Alg. 1 step 8; also the undivided backward-data pass of Alg. 1 step 9).
//
// Arithmetic, tile walk, K groups and epilogue are those of conv_stream_kernel.  What differs is who issues the
// direct-to-LDS loads.  A wave needs about 64 cycles to issue one 16-byte-per-lane buffer load to LDS and the
// few vector instructions that form its address, and it issues in order: in a kernel whose waves both load and
// multiply, a slab of a 128x128 tile costs a wave 5 loads = 320+ cycles during which it starts no MFMA, next to
// 512 cycles of MFMA work (measured: steps that carry loads take 300-500 cycles, the others about 100).  Here
// NP extra waves per workgroup do nothing but stage slabs (each handles every NP-th 1 KB load of a slab), and
// the WM*WN*KS compute waves never touch vector memory in the main loop: their instruction stream is MFMAs,
// fragment reads and code expansion only.  Hand-over per slab, as before, is one s_barrier: a load wave waits
// for its own loads of the next slab (s_waitcnt vmcnt) before it arrives, a compute wave arrives when it has
// finished the first half of the current slab; after the barrier the load waves refill the stage of the
// previous slab.  Four stages, so that a load has two slab times to land.
#include <mutex>

#include "twn_kernels.h"
#include "twn_lds_asm.h"
#include "twn_mfma.h"
#include "twn_stream_epilogue.h"

namespace twn {

#ifdef TWN_TRACE
// development build only: timestamps (shader clock) of one slab, 16 slots per workgroup
__device__ uint64_t* g_pc_trace = nullptr;
extern "C" int32_t twn_debug_set_pc_trace(void* buf) {
    uint64_t* p = static_cast<uint64_t*>(buf);
    return hipMemcpyToSymbol(HIP_SYMBOL(g_pc_trace), &p, sizeof(p)) == hipSuccess ? 0 : -6;
}
#define TWN_PTS(i) asm volatile("s_memtime %0" : "=s"(ts[i]))
// coarse timeline of a workgroup's first tiles: slots 16.. of 32
#define TWN_PCOARSE(slot)                                                                             \
    do {                                                                                              \
        if (trace_buf && tid == 0 && (slot) < 8)                                                     \
            trace_buf[static_cast<size_t>(blockIdx.x) * 32 + 16 + (slot)] = __builtin_readcyclecounter(); \
    } while (0)
#else
#define TWN_PTS(i) do {} while (0)
#define TWN_PCOARSE(slot) do {} while (0)
#endif

struct StreamPcArgs {
    GatherGemm g;
    FastDivU divOW, divOH;      // GEMM row -> (image, oh, ow)
    FastDivU divTN;             // tile -> (row block, column block)
    FastDivU divSPT, divS;      // K slab -> (tap, channel slab) -> (filter row, filter column)
    uint32_t x_bytes, w_bytes, y_bytes;  // sizes for the buffer descriptors
    uint32_t tiles, tiles_n;
    int32_t KT;                 // K / 64
    int32_t spt;                // 64-channel slabs per tap (IC / 64)
};

template <int BM, int BN, int WM, int WN, int STAGES, bool GEMM, int OCC, int KS, int NP>
// (the second launch bound is in waves per SIMD)
__global__ __launch_bounds__(64 * (WM * WN * KS + NP), (OCC * (WM * WN * KS + NP) + 3) / 4)
void conv_stream_pc_kernel(const StreamPcArgs a) {
    constexpr int NWG = WM * WN;                   // compute waves per K group
    constexpr int NWC = NWG * KS;                  // compute waves
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int A_BYTES = BM * 128;
    constexpr int B_BYTES = BN * 16;
    constexpr int SUB_BYTES = A_BYTES + B_BYTES;   // one slab of one K group
    constexpr int STAGE_BYTES = KS * SUB_BYTES;
    constexpr int PD = STAGES - 1;                 // slabs in flight ahead of the one being multiplied
    constexpr int LA = BM / 8, LB = BN / 64;       // 1 KB loads of one K group's slab: activation row blocks, code blocks
    constexpr int LG = LA + LB;
    constexpr int LTOT = KS * LG;
    constexpr int NLP = (LTOT + NP - 1) / NP;      // loads per load wave and slab (the last ones may be dummies)
    constexpr int EPI_CH = TN < 64 ? TN : 64;      // channels staged at a time
    constexpr int EPI_ROW = EPI_CH * 2 + 16;
    constexpr int EPI_WAVE = 32 * EPI_ROW;         // one block of 32 pixel rows per wave
    constexpr int RED_MI_FIT = STAGE_BYTES / (NWG * NI * 4096);
    constexpr int RED_MI = RED_MI_FIT < MI ? RED_MI_FIT : MI;
    static_assert(BM % 32 == 0 && BN % 64 == 0 && TN % 32 == 0 && TM % 32 == 0, "tile shape");
    static_assert(STAGES >= 3 && NP >= 1, "pipeline shape");
    static_assert(NWG * EPI_WAVE <= STAGE_BYTES, "epilogue staging must fit in one pipeline stage");
    static_assert(KS == 1 || (RED_MI >= 1 && MI % RED_MI == 0), "the reduction must fit in the free stage");
    static_assert(BN <= 64 * NWC, "one compute thread per column loads the column parameters");
    static_assert(MI <= 8 && NI <= 4, "fragment reads use immediate offsets");
    static_assert((PD - 1) * NLP < 64, "vmcnt is a 6-bit counter");
    // barriers of a tile's epilogue (every wave of the workgroup executes each of them)
    constexpr int EPI_BARRIERS = 1 + (KS > 1 ? 2 * (KS - 1) * (MI / RED_MI) : 0);

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    float* colbuf = reinterpret_cast<float*>(smem + STAGES * STAGE_BYTES);          // [2][2][BN]: mul, add of even / odd tiles
    unsigned char* dummy = smem + STAGES * STAGE_BYTES + 4 * BN * 4;                // 1 KB sink of the padding loads

    const GatherGemm& g = a.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#ifdef TWN_TRACE
    uint64_t* const trace_buf = g_pc_trace;
    TWN_PCOARSE(0);
#endif

    // ---- this workgroup's tiles (as in conv_stream_kernel: each XCD owns a contiguous range) ----
    const uint32_t G = gridDim.x, b = blockIdx.x;
    const uint32_t xcd = b & 7, j = b >> 3;
    const uint32_t gx = (G + 7 - xcd) >> 3;
    const uint32_t q = a.tiles >> 3, r = a.tiles & 7;
    const uint32_t count_x = q + (xcd < r ? 1u : 0u);
    const uint32_t start_x = xcd * q + (xcd < r ? xcd : r);
    if (j >= count_x) return;                               // whole workgroup, before any barrier
    const uint32_t n_my = (count_x - j + gx - 1) / gx;
    auto tile_id = [&](uint32_t i) __attribute__((always_inline)) -> uint32_t { return start_x + j + i * gx; };

    const int KT = a.KT;
    const int KTS = (KT + KS - 1) / KS;            // slabs per K group
    const uint32_t total = n_my * static_cast<uint32_t>(KTS);

    if (wave >= NWC) {
        // =================================== load wave ===================================
        auto producer = [&](auto p_tag) __attribute__((always_inline)) {
        constexpr int p = decltype(p_tag)::value;
        const __amdgpu_buffer_rsrc_t rx = make_rsrc(g.X, a.x_bytes), rw = make_rsrc(g.Wq, a.w_bytes);
        // load i of this wave is load l = p + NP*i of the slab: K group l / LG, then activation row block
        // (l % LG < LA) or code block.  LDS row r keeps logical 16-byte chunk c at position c ^ ((r >> 1) & 7):
        // the swizzle is applied by choosing which chunk of the row this lane fetches.
        uint32_t voff[NLP];          // activation block: offset of the row (GEMM) / of tap (0,0) (convolution); code block: row offset
        int ih0[NLP], iw0[NLP];
        auto tile_setup = [&](uint32_t t, bool valid) __attribute__((always_inline)) {
            const uint32_t tm = fdiv_u(t, a.divTN);
            const uint32_t tn = t - tm * a.tiles_n;
            const uint32_t m0 = tm * BM;
#pragma unroll
            for (int i = 0; i < NLP; ++i) {
                const int l = p + NP * i;
                const int within = l % LG;          // wave-uniform
                uint32_t vo = kBufOutside;
                int h0 = -(1 << 28), w0 = -(1 << 28);
                if (l < LTOT && valid) {
                    const int kc = (lane & 7) ^ ((within & 1) * 4 + ((lane >> 4) & 3));
                    if (within < LA) {
                        const uint32_t m = m0 + static_cast<uint32_t>(within * 8 + (lane >> 3));
                        if (GEMM) {
                            const uint32_t o = (m * static_cast<uint32_t>(g.xs) + static_cast<uint32_t>(kc * 8)) * 2u;
                            vo = (m < static_cast<uint32_t>(g.M)) ? o : kBufOutside;
                            h0 = w0 = 0;
                        } else {
                            const uint32_t tt = fdiv_u(m, a.divOW);
                            const int ow = static_cast<int>(m - tt * static_cast<uint32_t>(g.OW));
                            const uint32_t img = fdiv_u(tt, a.divOH);
                            const int oh = static_cast<int>(tt - img * static_cast<uint32_t>(g.OH));
                            const int hh = oh * g.sh - g.ph, ww = ow * g.sw - g.pw;
                            // 32-bit wrapping arithmetic: the true offset of every tap that passes the bounds test
                            // lies in [0, 2^31)
                            const uint32_t pix = (img * static_cast<uint32_t>(g.IH) + static_cast<uint32_t>(hh)) *
                                                     static_cast<uint32_t>(g.IW) + static_cast<uint32_t>(ww);
                            const bool rv = m < static_cast<uint32_t>(g.M);
                            vo = rv ? (pix * static_cast<uint32_t>(g.xs) + static_cast<uint32_t>(kc * 8)) * 2u : kBufOutside;
                            h0 = rv ? hh : -(1 << 28);
                            w0 = rv ? ww : -(1 << 28);
                        }
                    } else {
                        const uint32_t ncol = tn * BN + static_cast<uint32_t>((within - LA) * 64 + lane);
                        vo = (ncol < static_cast<uint32_t>(g.NC)) ? ncol * static_cast<uint32_t>(g.wpr) * 4u : kBufOutside;
                    }
                }
                voff[i] = vo;
                ih0[i] = h0;
                iw0[i] = w0;
            }
        };
        uint32_t lt = 0;
        int lk = 0;
        const int32_t strR = g.dh * g.IW * static_cast<int>(g.xs) * 2, strS = g.dw * static_cast<int>(g.xs) * 2;
        // the loads of this wave for stream position (tile lt, group slab lk) into `stage`
        auto issue = [&](int stage) __attribute__((always_inline)) {
            unsigned char* sbase = smem + stage * STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < NLP; ++i) {
                const int l = p + NP * i;
                const int kgl = l / LG, within = l % LG;       // wave-uniform
                if (l >= LTOT) {
                    buf_dma16(rx, kBufOutside, 0u, dummy);
                    continue;
                }
                const int sl = lk * KS + kgl;                   // K slab
                const bool in_k = sl < KT;
                unsigned char* dst = sbase + kgl * SUB_BYTES;
                if (within >= LA) {
                    buf_dma16(rw, in_k ? voff[i] : kBufOutside, static_cast<uint32_t>(sl) * 16u, dst + A_BYTES + (within - LA) * 1024);
                } else if (GEMM) {
                    buf_dma16(rx, in_k ? voff[i] : kBufOutside, static_cast<uint32_t>(sl) * 128u, dst + within * 1024);
                } else {
                    const uint32_t tap = fdiv_u(static_cast<uint32_t>(sl), a.divSPT);
                    const int c0 = (sl - static_cast<int>(tap) * a.spt) * 64;
                    const int rr = static_cast<int>(fdiv_u(tap, a.divS));
                    const int ss = static_cast<int>(tap) - rr * g.S;
                    const int32_t delta_b = rr * strR + ss * strS + c0 * 2;
                    const bool ok = (static_cast<unsigned>(ih0[i] + rr * g.dh) < static_cast<unsigned>(g.IH)) &
                                    (static_cast<unsigned>(iw0[i] + ss * g.dw) < static_cast<unsigned>(g.IW)) & in_k;
                    buf_dma16(rx, ok ? voff[i] + static_cast<uint32_t>(delta_b) : kBufOutside, 0u, dst + within * 1024);
                }
            }
            if (++lk == KTS) {
                lk = 0;
                ++lt;
                tile_setup(tile_id(lt), lt < n_my);
            }
        };

        tile_setup(tile_id(0), true);
#pragma unroll
        for (int s = 0; s < PD; ++s) issue(s % STAGES);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((PD - 1) * NLP));
        __builtin_amdgcn_s_barrier();                       // first slab landed
        int fill = PD % STAGES;
        int kt = 0;
        for (uint32_t s = 0; s < total; ++s) {
            // hand-over of slab s: the next slab has landed (the PD-2 younger ones may stay in flight)
#ifdef TWN_TRACE
            uint64_t ts[4];
#endif
            TWN_PTS(0);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(vmcnt_imm((PD - 2) * NLP));
            TWN_PTS(1);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            TWN_PTS(2);
            issue(fill);                                    // refill the stage of slab s-1
            TWN_PTS(3);
#ifdef TWN_TRACE
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (trace_buf && p == 0 && lane == 0 && s == 5)
                for (int i = 0; i < 4; ++i) trace_buf[static_cast<size_t>(blockIdx.x) * 32 + 8 + i] = ts[i];
#endif
            fill = (fill + 1 == STAGES) ? 0 : fill + 1;
            if (++kt == KTS) {
                kt = 0;
#pragma unroll
                for (int e = 0; e < EPI_BARRIERS; ++e) __builtin_amdgcn_s_barrier();
            }
        }
        // the trailing zero loads still target this workgroup's LDS: they must have landed before it ends
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        };
        static_for<NP>([&](auto p_tag) __attribute__((always_inline)) {
            if (wave - NWC == decltype(p_tag)::value) producer(p_tag);
        });
        return;
    }

    // =================================== compute wave ===================================
    const int kg = wave / NWG, wv = wave % NWG;    // K group, wave inside the group
    const int wm = wv / WN, wn = wv % WN;
    const int lrow = lane & 31, lh = lane >> 5;

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

    // One MFMA step (see gather_gemm_dma_kernel): fragment reads and code expansion of the next step are placed
    // between the MFMAs of this one; no vector-memory instruction in here.
    auto step = [&](auto kk_tag, auto cur_tag, int stage, int next) __attribute__((always_inline)) {
        constexpr int KK = decltype(kk_tag)::value;
        constexpr int CUR = decltype(cur_tag)::value;
        constexpr int NM = MI * NI;
        constexpr int SET = KK & 1, NSET = SET ^ 1;
        constexpr int KN = (KK + 1) & 3;
        constexpr int BSRC = (KK == 3) ? (CUR ^ 1) : CUR;
        constexpr int P_RA = MI;
        constexpr int P_RB = (KK == 2) ? 1 : 0;
        constexpr int P_D = 4 * NI;
        constexpr int P = P_RA + P_RB + P_D;
        const uint32_t a_addr = lds_base + ((KK == 3) ? next : stage) * STAGE_BYTES + aoff[KN];
        auto piece = [&](auto p_tag) __attribute__((always_inline)) {
            constexpr int pp = decltype(p_tag)::value;
            if constexpr (pp < P_RA) {
                lds_read128<pp * 32 * 128>(afrag[NSET][pp], a_addr);
            } else if constexpr (pp < P_RA + P_RB) {
                lds_read64_n<NI, 32 * 16>(breg[CUR ^ 1], lds_base + next * STAGE_BYTES + boff);
            } else {
                constexpr int qq = pp - P_RA - P_RB;
                expand(std::integral_constant<int, KN>{}, std::integral_constant<int, qq / 4>{},
                       std::integral_constant<int, qq % 4>{}, breg[BSRC], bfrag[NSET]);
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
                constexpr int pp = decltype(p_tag)::value;
                if constexpr (pp * NM / P == jj) piece(p_tag);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        lds_wait<0>();
        lds_ready<MI>(afrag[NSET]);
        if constexpr (KK == 2) lds_ready<NI>(breg[CUR ^ 1]);
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- epilogue of the tile the compute stream has just finished (as in conv_stream_kernel) ----
    const uint32_t ldyB = static_cast<uint32_t>(g.ldy) * 2u;
    TileStoreLane<EPI_CH> store_lane;
    store_lane.init(lane, ldyB);
    uint32_t ct = 0;
    auto epilogue = [&](int free_stage) __attribute__((always_inline)) {
#ifdef TWN_TRACE
        uint64_t es[4];
#define TWN_ES(i) do { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); asm volatile("s_memtime %0" : "=s"(es[i])); } while (0)
#else
#define TWN_ES(i) do {} while (0)
#endif
        TWN_ES(0);
        float* cmul = colbuf + (ct & 1u) * (2 * BN);
        float* cadd = cmul + BN;
        if (tid < BN) {
            cmul[tid] = 0.5f * cp_alpha * cp_scale;      // codes were +-2
            cadd[tid] = cp_shift;
        }
        // every wave has finished reading the stage of the last slab, and the column parameters are visible
        // (a bare s_barrier does not wait for this wave's LDS writes)
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        TWN_ES(1);
        if constexpr (KS > 1) {
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
        TWN_ES(2);
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
        TWN_ES(3);
#ifdef TWN_TRACE
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (trace_buf && tid == 0 && ct == 0)
            for (int i = 0; i < 4; ++i) trace_buf[static_cast<size_t>(blockIdx.x) * 32 + 24 + i] = es[i];
#endif
        acc_clear();
        ++ct;
        if (ct < n_my) colparam_load(tile_id(ct));
    };

    // ---- prologue: column parameters of the first tile; the load waves bring the first slab ----
    colparam_load(tile_id(0));
    acc_clear();
    TWN_PCOARSE(1);
    __builtin_amdgcn_s_barrier();                           // first slab landed (the load waves waited for it)
    asm volatile("" ::: "memory");
    TWN_PCOARSE(2);
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
    int kt = 0;             // slab of the current tile
    auto slab = [&](auto cur_tag) __attribute__((always_inline)) {
        const int next = (stage + 1 == STAGES) ? 0 : stage + 1;
#ifdef TWN_TRACE
        uint64_t ts[6];
#endif
        TWN_PTS(0);
        step(std::integral_constant<int, 0>{}, cur_tag, stage, next);
        TWN_PTS(1);
        step(std::integral_constant<int, 1>{}, cur_tag, stage, next);
        // hand-over: the load waves have seen the next slab land; the stage of the previous slab is free
        TWN_PTS(2);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        TWN_PTS(3);
        step(std::integral_constant<int, 2>{}, cur_tag, stage, next);
        TWN_PTS(4);
        step(std::integral_constant<int, 3>{}, cur_tag, stage, next);
        TWN_PTS(5);
#ifdef TWN_TRACE
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (trace_buf && tid == 0 && ct == 0 && kt == 5)
            for (int i = 0; i < 6; ++i) trace_buf[static_cast<size_t>(blockIdx.x) * 32 + i] = ts[i];
        if (trace_buf && tid == 0 && ct == 0 && kt == 6) trace_buf[static_cast<size_t>(blockIdx.x) * 32 + 6] = ts[0];
#endif
        const int done = stage;
        stage = next;
        if (++kt == KTS) {
            kt = 0;
            TWN_PCOARSE(3 + 2 * ct);
            epilogue(done);
            TWN_PCOARSE(2 + 2 * ct);      // ct was advanced by the epilogue
        }
    };
    for (uint32_t s = 0; s < total; s += 2) {
        slab(std::integral_constant<int, 0>{});
        if (s + 1 < total) slab(std::integral_constant<int, 1>{});
    }
}

// ---- host side ------------------------------------------------------------------------------------------

namespace {

int pc_num_cus() {
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

template <int BM, int BN, int WM, int WN, int STAGES, bool GEMM, int OCC, int KS, int NP>
int32_t launch_pc_kernel(const StreamPcArgs& a, hipStream_t st) {
    constexpr int SMEM = STAGES * KS * (BM * 128 + BN * 16) + 4 * BN * 4 + 1024;
    constexpr int THREADS = 64 * (WM * WN * KS + NP);
    static_assert(SMEM <= 160 * 1024, "LDS budget");
    static_assert(THREADS <= 1024, "workgroup size");
    auto k = conv_stream_pc_kernel<BM, BN, WM, WN, STAGES, GEMM, OCC, KS, NP>;
    static std::once_flag once;
    static int per_cu = 0;
    std::call_once(once, [&] {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, SMEM) !=
            hipSuccess)
            return;
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k, THREADS, SMEM) == hipSuccess && n > 0) per_cu = n;
    });
    if (per_cu <= 0) return TWN_ERR_HIP;
    int occ = per_cu;
    const int cap = env_int("TWN_STREAM_OCC", 0);
    if (cap > 0 && cap < occ) occ = cap;
    int64_t grid = static_cast<int64_t>(pc_num_cus()) * occ;
    if (grid > a.tiles) grid = a.tiles;
    k<<<dim3(static_cast<unsigned>(grid)), dim3(THREADS), SMEM, st>>>(a);
    return launch_status();
}

template <int BM, int BN, int WM, int WN, int STAGES, int OCC, int KS, int NP>
int32_t launch_pc_tile(const GatherGemm& g, hipStream_t st) {
    const int64_t tiles_n = (g.NC + BN - 1) / BN;
    const int64_t tiles = ((g.M + BM - 1) / BM) * tiles_n;
    if (tiles <= 0 || tiles >= (1LL << 31)) return TWN_ERR_SHAPE;
    StreamPcArgs a;
    a.g = g;
    a.divOW = make_fastdiv_u(static_cast<uint32_t>(g.OW));
    a.divOH = make_fastdiv_u(static_cast<uint32_t>(g.OH));
    a.divTN = make_fastdiv_u(static_cast<uint32_t>(tiles_n));
    a.spt = g.plain_gemm ? 1 : g.IC / 64;
    a.divSPT = make_fastdiv_u(static_cast<uint32_t>(a.spt));
    a.divS = make_fastdiv_u(static_cast<uint32_t>(g.S));
    const int64_t in_rows = g.plain_gemm ? g.M : (g.M / (static_cast<int64_t>(g.OH) * g.OW)) * g.IH * g.IW;
    a.x_bytes = static_cast<uint32_t>(((in_rows - 1) * g.xs + (g.plain_gemm ? g.K : g.IC)) * 2);
    a.w_bytes = static_cast<uint32_t>(static_cast<int64_t>(g.NC) * g.wpr * 4);
    a.y_bytes = static_cast<uint32_t>(((g.M - 1) * g.ldy + g.NC) * 2);
    a.tiles = static_cast<uint32_t>(tiles);
    a.tiles_n = static_cast<uint32_t>(tiles_n);
    a.KT = g.K / 64;
    return g.plain_gemm ? launch_pc_kernel<BM, BN, WM, WN, STAGES, true, OCC, KS, NP>(a, st)
                        : launch_pc_kernel<BM, BN, WM, WN, STAGES, false, OCC, KS, NP>(a, st);
}

}  // namespace

// Same tile ids and applicability (conv_stream_applicable) as launch_conv_stream; `ks` K groups (1 or 2), `np`
// load waves (2 or 4), `stages` 3 or 4.
int32_t launch_conv_stream_pc(const GatherGemm& g, int tile, int ks, int np, int stages, hipStream_t st) {
    const int key = tile * 1000 + ks * 100 + np * 10 + stages;
    switch (key) {
        case 14124: return launch_pc_tile<64, 128, 1, 4, 4, 3, 1, 2>(g, st);
        case 14144: return launch_pc_tile<64, 128, 1, 4, 4, 2, 1, 4>(g, st);
        case 14244: return launch_pc_tile<64, 128, 1, 4, 4, 1, 2, 4>(g, st);
        case 15144: return launch_pc_tile<128, 128, 1, 4, 4, 2, 1, 4>(g, st);
        case 16144: return launch_pc_tile<128, 64, 2, 2, 4, 2, 1, 4>(g, st);
        case 17144: return launch_pc_tile<128, 256, 1, 4, 4, 1, 1, 4>(g, st);
        default: return TWN_ERR_UNSUPPORTED;
    }
}

}  // namespace twn
