// 3x3 stride-1 ternary convolution over 64 input channels with the weights resident in registers, gfx950
// (Eq. 2, Alg. 1 step 8; with the transposed codes and mirrored taps the backward-data pass of the same layers,
// Alg. 1 step 9).
//
// With 64 output channels per tile the slab pipeline of the generic kernels spends as many cycles issuing its
// gathered loads (every activation is fetched once per tap: nine times) and expanding the same 2-bit codes again
// for every tile as it spends in the matrix cores.  This kernel removes both:
//   * K = 9 * 64 = 576 is small enough for the expanded weights to live in registers: a wave owns 32 output
//     channels, and its 36 weight fragments (144 registers) are built ONCE per workgroup, straight from the packed
//     2-bit rows in global memory.  The main loop has no code expansion and no weight traffic at all;
//   * persistent workgroups walk 8x8 tiles of output pixels; the 10x10 input patch (tile + halo) is read ONCE from
//     global memory (the patch of tile i+2 is requested during tile i and is in flight in registers while tile i+1
//     is multiplied) and all nine taps read their shifted windows of it from LDS.  A patch pixel takes 144 bytes and a patch row 1664
//     bytes in LDS, which makes every 16-lane group of a fragment read (two tile rows of eight pixels) hit 16
//     different 16-byte bank groups for every tap, and makes the tap and channel-chunk part of a fragment's
//     address a compile-time constant: one address register, the rest sits in the read's immediate offset;
//   * per MFMA the loop issues one 16-byte LDS read and nothing else.
// The epilogue (alpha/2, scale, shift, residual, ReLU, one rounding, transposition through LDS, 16-byte stores)
// is that of the other contraction kernels.  No workspace, no preparation launch.
#include <cstdlib>
#include <mutex>

#include "twn_kernels.h"
#include "twn_lds_asm.h"

namespace twn {

constexpr int kC64Tile = 8;                     // output pixels per tile side
constexpr int kC64PSide = kC64Tile + 2;         // patch side (tile + halo of a 3x3 filter)
constexpr int kC64PixB = 144;                   // LDS bytes per patch pixel: 128 + 16 (odd multiple of 16)
constexpr int kC64RowB = 1664;                  // LDS bytes per patch row: >= 10 * 144 and = 8 (mod 16) in 16-byte units
constexpr int kC64Patch = kC64PSide * kC64RowB; // 16640
constexpr int kC64Stg = 4 * 32 * 80;            // epilogue staging: 32 pixel rows x (32 channels + pad) per wave
constexpr int kC64Chunks = kC64PSide * kC64PSide * 8;   // 16-byte chunks of a patch (800)
constexpr int kC64Nit = (kC64Chunks + 255) / 256;       // chunks per lane (4)
constexpr int kC64Steps = 36;                   // MFMA steps: 9 taps x 4 groups of 16 channels
constexpr int kC64Smem = 2 * kC64Patch + kC64Stg + 2 * 64 * 4;

struct C64Args {
    const uint16_t* X;
    const uint32_t* Wq;
    const float* alpha;
    const float* scale;
    const float* shift;
    const uint16_t* residual;
    uint16_t* Y;
    int32_t H, W, NC, P, Q;         // input image, output channels, output image
    int32_t y0off, x0off;           // patch origin = (p0 + y0off, q0 + x0off)
    int32_t wpr, rows_per_group, relu;
    int32_t ldy;
    uint32_t tiles, tiles_x, tiles_y;
    FastDivU divTX, divTY;
    uint32_t x_bytes, y_bytes;      // sizes of X and of the output / residual tensor
};

// FLIP: the taps run against the pixel order (backward-data: input row = output row + pad - r)
// RES: a residual tensor is added (its values for a tile are requested before the tile's MFMA loop)
template <bool FLIP, bool RES>
__global__ __launch_bounds__(256, 2) void conv_c64_kernel(const C64Args a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    unsigned char* stg_base = smem + 2 * kC64Patch;
    float* colmul = reinterpret_cast<float*>(stg_base + kC64Stg);     // [64] 0.5*alpha*scale
    float* coladd = colmul + 64;                                       // [64] shift

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lh = lane >> 5;
    const int n0 = static_cast<int>(blockIdx.y) * 64;

    if (tid < 64) {
        const int ncol = n0 + tid;
        const int ag = (a.rows_per_group >= a.NC) ? 0 : ncol / a.rows_per_group;
        colmul[tid] = 0.5f * a.alpha[ag] * (a.scale ? a.scale[ncol] : 1.0f);     // codes become +-2
        coladd[tid] = a.shift ? a.shift[ncol] : 0.0f;
    }

    // ---- this workgroup's tiles: each XCD owns a contiguous range (neighbouring patches share halos in its L2) ----
    const uint32_t G = gridDim.x, b = blockIdx.x;
    const uint32_t xcd = b & 7, j = b >> 3;
    const uint32_t gx = (G + 7 - xcd) >> 3;
    const uint32_t q8 = a.tiles >> 3, r8 = a.tiles & 7;
    const uint32_t count_x = q8 + (xcd < r8 ? 1u : 0u);
    const uint32_t start_x = xcd * q8 + (xcd < r8 ? xcd : r8);
    if (j >= count_x) return;
    const uint32_t n_my = (count_x - j + gx - 1) / gx;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.X, a.x_bytes);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.Y, a.y_bytes);
    const __amdgpu_buffer_rsrc_t rr_desc = make_rsrc(RES ? a.residual : a.X, RES ? a.y_bytes : 0u);
    struct Tile {
        int img, p0, q0;
    };
    auto tile_of = [&](uint32_t i) __attribute__((always_inline)) -> Tile {
        uint32_t t = start_x + j + i * gx;
        uint32_t u = fdiv_u(t, a.divTX);
        const int tx = static_cast<int>(t - u * a.tiles_x);
        t = u;
        u = fdiv_u(t, a.divTY);
        const int ty = static_cast<int>(t - u * a.tiles_y);
        return Tile{static_cast<int>(u), ty * kC64Tile, tx * kC64Tile};
    };

    // patch of a tile -> registers: lane handles the 16-byte chunks tid, tid + 256, ... (pixel = chunk / 8).  Which
    // patch chunk a lane handles never changes: its coordinates and offsets are computed once.
    int py[kC64Nit], px[kC64Nit];               // patch row and column of the chunk's pixel (far negative: no chunk)
    uint32_t goff[kC64Nit];                     // byte offset of the chunk relative to the patch origin in X
    uint32_t loff[kC64Nit];                     // byte offset in the LDS patch
    bool has[kC64Nit];
#pragma unroll
    for (int it = 0; it < kC64Nit; ++it) {
        const int ci = it * 256 + tid;
        const int pl = ci >> 3, c = ci & 7;
        const int y = pl / kC64PSide, x = pl - y * kC64PSide;
        has[it] = ci < kC64Chunks;
        py[it] = has[it] ? y : -(1 << 24);
        px[it] = x;
        goff[it] = (static_cast<uint32_t>(y) * static_cast<uint32_t>(a.W) + static_cast<uint32_t>(x)) * 128u + c * 16u;
        loff[it] = static_cast<uint32_t>(y * kC64RowB + x * kC64PixB + c * 16);
    }
    u32x4 pr[kC64Nit];
    auto load_patch = [&](const Tile& t, bool live) __attribute__((always_inline)) {
        const int y0 = t.p0 + a.y0off, x0 = t.q0 + a.x0off;
        // 32-bit wrapping arithmetic: the offset of every chunk that lies inside the image is in [0, x_bytes);
        // a chunk outside the image (the zero border) gets an offset past the descriptor and reads zeros
        const uint32_t base = ((static_cast<uint32_t>(t.img) * a.H + static_cast<uint32_t>(y0)) * a.W + static_cast<uint32_t>(x0)) * 128u;
#pragma unroll
        for (int it = 0; it < kC64Nit; ++it) {
            const bool ok = live & (static_cast<unsigned>(y0 + py[it]) < static_cast<unsigned>(a.H)) &
                            (static_cast<unsigned>(x0 + px[it]) < static_cast<unsigned>(a.W));
            pr[it] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? base + goff[it] : kBufOutside, 0, 0));
        }
    };
    auto store_patch = [&](unsigned char* buf) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < kC64Nit; ++it)
            if (has[it]) *reinterpret_cast<u32x4*>(buf + loff[it]) = pr[it];
    };

    // per-lane fragment base inside a patch: pixel (tile row wm*4 + (lrow >> 3), tile column lrow & 7), k half lh
    const int pbase = (wm * 4 + (lrow >> 3)) * kC64RowB + (lrow & 7) * kC64PixB + lh * 16;

    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) unsigned char*)smem));
    typedef short s16x2 __attribute__((ext_vector_type(2)));
    const s16x2 floor2 = __builtin_bit_cast(s16x2, a.relu ? 0u : 0x80008000u);
    f32x16 acc;
    unsigned char* stg = stg_base + wave * (32 * 80);
    // read-back lane (it): staged row it*16 + lane/4 = tile pixel (wm*4 + row/8, row%8), 16-byte chunk lane&3;
    // its byte offset in Y relative to the tile's first pixel and channel n0
    uint32_t yoff[2];
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int row = it * 16 + (lane >> 2);
        yoff[it] = ((static_cast<uint32_t>(wm * 4 + (row >> 3)) * a.Q + static_cast<uint32_t>(row & 7)) * a.ldy +
                    static_cast<uint32_t>(wn * 32 + (lane & 3) * 8)) * 2u;
    }

    // Order of the vector-memory operations per tile i: MFMA loop; wait for everything in flight; patch i+1
    // registers -> LDS; request patch i+2; epilogue arithmetic; request the residual values of tile i+1; output
    // stores of tile i; barrier.  The one wait of an iteration sits behind a whole MFMA loop, so the stores it
    // covers (tile i-1) have had a tile's time to complete.
    auto load_residual = [&](const Tile& t, u32x2* dst, bool live) __attribute__((always_inline)) {
        // accumulator layout: lane (pixel, k half lh) adds to channels q4*8 + lh*4 .. + 3
        const int p = t.p0 + wm * 4 + (lrow >> 3), q = t.q0 + (lrow & 7);
        const bool pix_ok = live & (p < a.P) & (q < a.Q);
        const uint32_t ro = ((static_cast<uint32_t>(t.img) * a.P + static_cast<uint32_t>(p)) * a.Q + static_cast<uint32_t>(q)) *
                                static_cast<uint32_t>(a.ldy) * 2u + static_cast<uint32_t>(n0 + wn * 32 + lh * 4) * 2u;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
            dst[q4] = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(rr_desc, pix_ok ? ro + q4 * 16u : kBufOutside, 0, 0));
    };
    Tile cur = tile_of(0);
    load_patch(cur, true);      // in flight while the weight fragments are built

    // ---- once per workgroup: the weight fragments of this wave's 32 channels, all 36 steps -------------------
    // Step ks covers k = 16 ks .. 16 ks + 15, i.e. packed word ks of the channel's row; lane (channel lrow, half lh)
    // holds k = 16 ks + 8 lh + 0..7 as four bf16 pairs.  Pair v is (even k: low half-word field 4 lh + v, odd k:
    // high half-word field 4 lh + v); a 2-bit field moved to bits [14,15] of a bf16 is 0 / +2.0 / -2.0.
    u32x4 bfrag[kC64Steps];
    {
        const uint32_t* row = a.Wq + static_cast<int64_t>(n0 + wn * 32 + lrow) * a.wpr;
        const int sh0 = 8 * lh;
#pragma unroll
        for (int j = 0; j < kC64Steps / 4; ++j) {
            const u32x4 w4 = *reinterpret_cast<const u32x4*>(row + 4 * j);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t w = w4[u] >> sh0;
#pragma unroll
                for (int v = 0; v < 4; ++v) bfrag[4 * j + u][v] = ((w >> (2 * v)) & 0x00030003u) << 14;
            }
        }
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    store_patch(smem);
    // Every request of the loop is issued unconditionally (a tile past the end of the walk gets offsets outside the
    // descriptor: no memory traffic, zeros back): straight-line code without divergent paths around the requests.
    Tile nxt = tile_of(1);
    load_patch(nxt, n_my > 1);
    u32x2 rres[4];
    if constexpr (RES) load_residual(cur, rres, true);
    // the first patch and the column parameters are in LDS (a bare barrier: the requests just issued stay in flight)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    int buf = 0;
    for (uint32_t i = 0; i < n_my; ++i) {
        const bool more = (i + 1 < n_my), more2 = (i + 2 < n_my);
        const uint32_t pb = lds_base + static_cast<uint32_t>(buf * kC64Patch + pbase);
        {
            // Step ks = tap * 4 + cq reads the 16 channels 16 cq .. 16 cq + 15 of the pixel one tap away: the whole
            // offset is an immediate.  The reads run AHEAD steps in front of the MFMAs through a ring of RING
            // registers (inline assembly with exact lgkmcnt waits: LDS operations complete in issue order); the
            // read of step ks + AHEAD lands in the registers of step ks - 1.
            constexpr int AHEAD = 8, RING = 9;
            u32x4 af[RING];
            auto read_step = [&](auto ks_tag) __attribute__((always_inline)) {
                constexpr int ks = decltype(ks_tag)::value;
                constexpr int t = ks >> 2, cq = ks & 3;
                constexpr int r = t / 3, s = t - 3 * r;
                constexpr int ro = FLIP ? 2 - r : r, co = FLIP ? 2 - s : s;
                lds_read128<ro * kC64RowB + co * kC64PixB + cq * 32>(af[ks % RING], pb);
            };
            static_for<AHEAD>(read_step);
            static_for<kC64Steps>([&](auto ks_tag) __attribute__((always_inline)) {
                constexpr int ks = decltype(ks_tag)::value;
                if constexpr (ks + AHEAD < kC64Steps) read_step(std::integral_constant<int, ks + AHEAD>{});
                constexpr int last = (ks + AHEAD < kC64Steps) ? ks + AHEAD : kC64Steps - 1;      // youngest read issued
                lds_wait<last - ks>();
                lds_ready<1>(&af[ks % RING]);
                // the first step starts from a zero C operand (an inline constant): no clearing pass
                const f32x16 c_in = (ks == 0) ? f32x16{} : acc;
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfrag[ks]),
                                                              __builtin_bit_cast(bf16x8, af[ks % RING]), c_in, 0, 0, 0);
            });
        }
        // Everything this wave has requested so far (patch i+1, the residual values of tile i, the stores of tile
        // i-1) is complete before the registers are used: one full wait instead of counted ones.  Counted waits
        // would rest on requests being answered in issue order also when all lanes of a request fall outside the
        // tensor and no memory is touched; the full wait needs no such assumption and sits behind a whole MFMA
        // loop, so it costs nothing measurable with two workgroups per CU.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        store_patch(smem + (buf ^ 1) * kC64Patch);
        const Tile nn = tile_of(i + 2);
        load_patch(nn, more2);
        // ---- epilogue: accumulator element e in this lane: tile pixel (wm*4 + (lrow>>3), lrow & 7),
        // channel wn*32 + (e>>2)*8 + lh*4 + (e&3) ----
        {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int nl = wn * 32 + q4 * 8 + lh * 4;
                const f32x4 mul = *reinterpret_cast<const f32x4*>(colmul + nl);
                const f32x4 add = *reinterpret_cast<const f32x4*>(coladd + nl);
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[q4 * 4 + e] * mul[e] + add[e];
                if constexpr (RES) {
                    const u32x2 rr = rres[q4];
                    v[0] += __uint_as_float(rr[0] << 16);
                    v[1] += __uint_as_float(rr[0] & 0xFFFF0000u);
                    v[2] += __uint_as_float(rr[1] << 16);
                    v[3] += __uint_as_float(rr[1] & 0xFFFF0000u);
                }
                // ReLU on the rounded pair: a packed signed 16-bit maximum against 0 (negative bf16 values are negative
                // as integers), or against the int16 minimum when there is no ReLU
                u32x2 pk;
                pk[0] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pack_bf16x2(v[0], v[1])), floor2));
                pk[1] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pack_bf16x2(v[2], v[3])), floor2));
                *reinterpret_cast<u32x2*>(stg + lrow * 80 + (q4 * 8 + lh * 4) * 2) = pk;
            }
        }
        if constexpr (RES) load_residual(nxt, rres, more);
        // same wave wrote and reads: LDS executes a wave's operations in order
        {
            u32x4 val[2];
#pragma unroll
            for (int it = 0; it < 2; ++it) val[it] = *reinterpret_cast<const u32x4*>(stg + (it * 16 + (lane >> 2)) * 80 + (lane & 3) * 16);
            const uint32_t ytile = (((static_cast<uint32_t>(cur.img) * a.P + static_cast<uint32_t>(cur.p0)) * a.Q +
                                     static_cast<uint32_t>(cur.q0)) * static_cast<uint32_t>(a.ldy) + static_cast<uint32_t>(n0)) * 2u;   // wave-uniform
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = it * 16 + (lane >> 2);
                const bool ok = (cur.p0 + wm * 4 + (row >> 3) < a.P) & (cur.q0 + (row & 7) < a.Q);
                // no scalar-offset field (the compiler adds no wait state after that form of a 16-byte store, and an
                // overwrite of the data registers in the next instruction then reaches memory)
                __builtin_amdgcn_raw_buffer_store_b128(val[it], ry, ok ? yoff[it] + ytile : kBufOutside, 0, kStoreThrough);
            }
        }
        // The next patch is complete (this wave's LDS writes have landed) and every wave is done with the current
        // one.  A bare barrier: __syncthreads() would also wait for the epilogue's global stores, i.e. for a
        // write round trip to memory per tile.
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        buf ^= 1;
        cur = nxt;
        nxt = nn;
    }
}

// ---- host side ------------------------------------------------------------------------------------------

static bool c64_plan(const GatherGemm& g, C64Args* a) {
    if (g.IC != 64 || g.xs != 64 || g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.divh != 1 || g.divw != 1) return false;
    if (!((g.dh == 1 && g.dw == 1) || (g.dh == -1 && g.dw == -1))) return false;
    if (g.y_f32 || g.plain_gemm || g.chunk_gather || g.orU != 0 || g.splits > 1) return false;
    if (g.NC % 64 != 0 || g.ldy % 8 != 0 || g.ldy >= (1 << 24) || g.OH < 1 || g.OW < 1) return false;
    if (g.M % (static_cast<int64_t>(g.OH) * g.OW) != 0) return false;
    const int64_t n_img = g.M / (static_cast<int64_t>(g.OH) * g.OW);
    const int64_t xb = n_img * g.IH * g.IW * 128;
    if (xb <= 0 || xb >= (1LL << 31)) return false;
    if (!aligned(g.X, 16) || !aligned(g.Wq, 16) || !aligned(g.Y, 16) || (g.residual && !aligned(g.residual, 8))) return false;
    if (g.wpr < kC64Steps) return false;
    // every patch pixel of a tile that holds an output pixel must be addressable relative to the patch origin
    if (std::abs(g.ph) > 8 || std::abs(g.pw) > 8) return false;
    a->X = static_cast<const uint16_t*>(g.X);
    a->Wq = static_cast<const uint32_t*>(g.Wq);
    a->alpha = g.alpha; a->scale = g.scale; a->shift = g.shift;
    a->residual = static_cast<const uint16_t*>(g.residual);
    a->Y = static_cast<uint16_t*>(g.Y);
    a->H = g.IH; a->W = g.IW; a->NC = g.NC; a->P = g.OH; a->Q = g.OW;
    // input row of tap r for output row p: p - ph + r*dh; the patch starts at the smallest of them
    a->y0off = -g.ph + (g.dh < 0 ? -2 : 0);
    a->x0off = -g.pw + (g.dw < 0 ? -2 : 0);
    a->wpr = g.wpr; a->rows_per_group = g.rows_per_group; a->relu = g.relu;
    a->ldy = static_cast<int32_t>(g.ldy);
    a->tiles_x = static_cast<uint32_t>((g.OW + kC64Tile - 1) / kC64Tile);
    a->tiles_y = static_cast<uint32_t>((g.OH + kC64Tile - 1) / kC64Tile);
    const int64_t tiles = n_img * a->tiles_x * a->tiles_y;
    if (tiles <= 0 || tiles >= (1LL << 30)) return false;
    a->tiles = static_cast<uint32_t>(tiles);
    a->divTX = make_fastdiv_u(a->tiles_x);
    a->divTY = make_fastdiv_u(a->tiles_y);
    a->x_bytes = static_cast<uint32_t>(xb);
    const int64_t yb = g.M * g.ldy * 2;
    if (yb >= (1LL << 31)) return false;
    a->y_bytes = static_cast<uint32_t>(yb);
    return true;
}

bool conv_c64_applicable(const GatherGemm& g) {
    C64Args a;
    return c64_plan(g, &a);
}

int32_t launch_conv_c64(const GatherGemm& g, hipStream_t st) {
    C64Args a;
    if (!c64_plan(g, &a)) return TWN_ERR_UNSUPPORTED;
    using Kern = void (*)(const C64Args);
    static const Kern kerns[4] = {conv_c64_kernel<false, false>, conv_c64_kernel<false, true>,
                                  conv_c64_kernel<true, false>, conv_c64_kernel<true, true>};
    const Kern k = kerns[(g.dh < 0 ? 2 : 0) + (g.residual ? 1 : 0)];
    static std::once_flag once;
    static int cus = 256;
    static bool allowed = false;
    std::call_once(once, [] {
        int dev = 0;
        hipDeviceProp_t p;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess && p.multiProcessorCount > 0)
            cus = p.multiProcessorCount;
        allowed = true;
        for (Kern kk : kerns)
            allowed = allowed && hipFuncSetAttribute(reinterpret_cast<const void*>(kk),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, kC64Smem) == hipSuccess;
    });
    if (!allowed) return TWN_ERR_HIP;
    const unsigned tiles_n = static_cast<unsigned>(g.NC / 64);
    int per_cu = 2;
    const int cap = env_int("TWN_C64_OCC", 0);
    if (cap > 0 && cap < per_cu) per_cu = cap;
    int64_t gx = static_cast<int64_t>(cus) * per_cu / tiles_n;
    if (gx < 8) gx = 8;
    if (gx > a.tiles) gx = a.tiles;
    k<<<dim3(static_cast<unsigned>(gx), tiles_n), dim3(256), kC64Smem, st>>>(a);
    return launch_status();
}

}  // namespace twn
