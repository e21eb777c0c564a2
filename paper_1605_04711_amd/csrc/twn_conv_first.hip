// First-layer ternary convolution (three input channels) on gfx950 (Eq. 2, Alg. 1 step 8).
//
// A layer with C = 3 has K = R*S*3 (27 for 3x3, 147 for the 7x7 stem): far too shallow for the slab pipeline
// of the generic kernels, and its NHWC pixels are 6 bytes, so no 16-byte chunk of a filter row is aligned.
// This kernel is built around those two facts:
//   * persistent workgroups walk 8x16 tiles of output pixels; for each tile the input patch with its halo
//     ((8-1)*stride+R rows) is read ONCE from global memory, two pixels (12 bytes, dword aligned because
//     patches start at even columns) per lane, widened to 4 channels on the way into LDS (8 bytes per pixel:
//     every tap pair is then one aligned 16-byte fragment), and the patch of tile i+2 is requested
//     during tile i (in flight in registers while tile i+1 is multiplied);
//   * K is re-ordered to (filter row, tap, 4 channels) with the taps of a row padded to a multiple of four
//     (7 -> 8 for the stem, 3 -> 4 for 3x3): one MFMA step covers four taps of one filter row.  The codes of
//     the phantom tap / channel are zero.  The whole expanded weight tile of a wave (32 channels x all K:
//     at most 14 steps x 4 registers) is built once per workgroup, straight from the packed 2-bit rows, and
//     stays in registers: the main loop has no code expansion and no weight traffic at all;
//   * the epilogue (alpha/2, scale, shift, residual, ReLU, one rounding, transposition through LDS, 16-byte
//     stores) is that of the other contraction kernels.
// Nothing is prepared in a separate launch and no workspace is used.
#include <mutex>
#include <type_traits>

#include "twn_kernels.h"
#include "twn_mfma.h"

namespace twn {

constexpr int kFirstTH = 8, kFirstTW = 16;      // output pixels of a tile
constexpr int kFirstStg = 4 * 64 * 80;          // epilogue staging: 64 pixel rows x (32 channels + pad) per wave

struct FirstArgs {
    const uint16_t* X;
    const uint32_t* Wq;
    const float* alpha;
    const float* scale;
    const float* shift;
    const uint16_t* residual;
    uint16_t* Y;
    int32_t N, H, W, O, R, S, sh, sw, ph, pw, P, Q;
    int32_t wpr, rows_per_group, relu;
    int32_t xoff;               // 0/1: the patch starts one column left of the first tap so that it starts at an even column
    int32_t kpr, ktot;          // MFMA steps per filter row (four taps each) and in total
    int32_t PH, PW, pairs;      // patch rows, columns (even), pixel pairs per patch row
    int32_t patch_bytes;        // PH*PW*8 rounded up to 16
    int32_t nit;                // pixel pairs per lane and patch = ceil(PH*pairs / 256)
    int32_t stagger;            // start delay per residency slot, in units of 512 cycles
    uint32_t tiles, tiles_x, tiles_y;
    FastDivU divTX, divTY, divPairs, divKq;
    uint32_t x_bytes, y_bytes;
    int32_t through;            // 1: output stores are written through (sc1)
};

typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));

#ifdef TWN_TRACE
// development build only: per-workgroup phase timestamps (shader clock), 16 slots per workgroup
__device__ uint64_t* g_first_trace = nullptr;
#define TWN_FTRACE(slot)                                                                                  \
    do {                                                                                                  \
        if (g_first_trace && threadIdx.x == 0 && (slot) < 16)                                             \
            g_first_trace[static_cast<size_t>(blockIdx.x) * 16 + (slot)] = __builtin_readcyclecounter();  \
    } while (0)
extern "C" int32_t twn_debug_set_first_trace(void* buf) {
    uint64_t* p = static_cast<uint64_t*>(buf);
    return hipMemcpyToSymbol(HIP_SYMBOL(g_first_trace), &p, sizeof(p)) == hipSuccess ? 0 : -6;
}
#else
#define TWN_FTRACE(slot) do {} while (0)
#endif

// EVEN_SW: the column stride is even, so every fragment is 16-byte aligned in the patch (one 16-byte read)
template <int KMAX, int NITMAX, bool EVEN_SW>
__global__ __launch_bounds__(256, 3) void conv_first_kernel(const FirstArgs a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    TWN_FTRACE(0);
    unsigned char* stg_base = smem + 2 * a.patch_bytes;
    float* colmul = reinterpret_cast<float*>(stg_base + kFirstStg);     // [64] 0.5*alpha*scale
    float* coladd = colmul + 64;                                          // [64] shift
    uint32_t* wl = reinterpret_cast<uint32_t*>(coladd + 64);              // [64][wpr] packed rows of this channel tile

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lh = lane >> 5;
    const int n0 = static_cast<int>(blockIdx.y) * 64;

    // ---- once per workgroup: column parameters and packed rows of its 64 channels -> LDS ----
    // the 64 packed rows of this channel tile are contiguous in memory: a flat copy, 16 bytes per lane and load
    {
        const int64_t first = static_cast<int64_t>(n0) * a.wpr, limit = static_cast<int64_t>(a.O) * a.wpr;
        for (int i = tid * 4; i < 64 * a.wpr; i += 1024) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (first + i < limit) v = *reinterpret_cast<const u32x4*>(a.Wq + first + i);
            *reinterpret_cast<u32x4*>(wl + i) = v;
        }
    }
    TWN_FTRACE(9);
    if (tid < 64) {
        const int ncol = n0 + tid;
        float mul = 0.0f, add = 0.0f;
        if (ncol < a.O) {
            const int ag = (a.rows_per_group >= a.O) ? 0 : ncol / a.rows_per_group;
            mul = 0.5f * a.alpha[ag] * (a.scale ? a.scale[ncol] : 1.0f);     // codes become +-2
            add = a.shift ? a.shift[ncol] : 0.0f;
        }
        colmul[tid] = mul;
        coladd[tid] = add;
    }
    __syncthreads();
    TWN_FTRACE(10);

    // ---- the weight tile of the workgroup, expanded once, cooperatively: W'[ch][k'] bf16 (+-2 / 0) in LDS with
    // k' = ((r*kpr + h)*4 + t)*4 + c (filter row, tap group, tap slot t = s + xoff - 4h, channel; zero where the
    // slot is no tap or c = 3).  The fragment of step ks = r*kpr + h for lane (channel, k half lh) is then the 16
    // bytes at k' = ks*16 + lh*8: one read per step.  The table lives where the patches and the staging rows
    // will be (it is dead once every lane holds its fragments).
    u32x4 bfrag[KMAX];
    {
        const int kq = a.ktot * 8;                       // dwords (bf16 pairs) per channel
        uint32_t* wt = reinterpret_cast<uint32_t*>(smem);
        const int slots = 4 * a.kpr;
        // One lane builds whole filter rows of one channel: the S*3 codes of row r are consecutive in k, so they
        // are pulled out of the packed words as ONE bit window (the words keep even k in the low and odd k in the
        // high half-word: spreading both halves to every second 2-bit group puts the 16 codes of a word in k
        // order), and every tap slot is then a 6-bit field of that window.
        auto spread = [](uint32_t x) __attribute__((always_inline)) -> uint32_t {      // 2-bit group i -> bits [4i, 4i+1]
            x = (x | (x << 8)) & 0x00FF00FFu;
            x = (x | (x << 4)) & 0x0F0F0F0Fu;
            x = (x | (x << 2)) & 0x33333333u;
            return x;
        };
        auto linear = [&](uint32_t word) __attribute__((always_inline)) -> uint32_t {
            return spread(word & 0xFFFFu) | (spread(word >> 16) << 2);
        };
        {
            const int ch = tid & 63;
            const uint32_t* row = wl + ch * a.wpr;
            for (int r = tid >> 6; r < a.R; r += 4) {
                const int k0 = r * a.S * 3;
                const int j0 = k0 >> 4, sh = (k0 & 15) * 2;
                const uint64_t l0 = linear(row[j0]), l1 = linear(row[j0 + 1]), l2 = linear(row[j0 + 2]);   // wpr >= j0 + 3
                const uint64_t low = l0 | (l1 << 32);
                const uint64_t win = (low >> sh) | (sh ? (l2 << (64 - sh)) : 0ull);      // codes k0, k0+1, ... from bit 0
                for (int t = 0; t < slots; ++t) {
                    const int sp = t - a.xoff;
                    uint32_t d0 = 0u, d1 = 0u;
                    if (sp >= 0 && sp < a.S) {                                           // wave-uniform
                        const uint32_t e = static_cast<uint32_t>(win >> (6 * sp)) & 0x3Fu;
                        // a 2-bit field moved to bits [14,15] of a bf16 is 0 / +2.0 / -2.0
                        d0 = ((e & 3u) << 14) | (((e >> 2) & 3u) << 30);
                        d1 = ((e >> 4) & 3u) << 14;
                    }
                    *reinterpret_cast<u32x2*>(wt + ch * kq + (r * slots + t) * 2) = u32x2{d0, d1};
                }
            }
        }
        __syncthreads();
        const unsigned char* mine = smem + (wn * 32 + lrow) * (kq * 4) + lh * 16;
#pragma unroll
        for (int ks = 0; ks < KMAX; ++ks)
            bfrag[ks] = (ks < a.ktot) ? *reinterpret_cast<const u32x4*>(mine + ks * 32) : u32x4{0u, 0u, 0u, 0u};
        __syncthreads();        // every lane has its fragments: the region may be overwritten by the first patch
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
        return Tile{static_cast<int>(u), ty * kFirstTH, tx * kFirstTW};
    };

    // patch of a tile -> registers: lane handles pixel pairs tid, tid + 256, ... (12 bytes each).  Which patch
    // pixel a lane handles never changes: its coordinates and offsets are computed once.
    int py[NITMAX], px[NITMAX];             // patch row and column of the pair (far negative: the lane has no pair)
    uint32_t goff[NITMAX];                  // byte offset of the pair relative to the patch origin in X
    uint32_t loff[NITMAX];                  // byte offset in the LDS patch
    bool has[NITMAX];
#pragma unroll
    for (int it = 0; it < NITMAX; ++it) {
        const uint32_t pi = static_cast<uint32_t>(it * 256 + tid);
        const uint32_t y = fdiv_u(pi, a.divPairs);
        const int xp = static_cast<int>(pi - y * a.pairs);
        has[it] = y < static_cast<uint32_t>(a.PH);
        py[it] = has[it] ? static_cast<int>(y) : -(1 << 24);
        px[it] = 2 * xp;
        goff[it] = (y * static_cast<uint32_t>(a.W) + static_cast<uint32_t>(2 * xp)) * 6u;
        loff[it] = (y * static_cast<uint32_t>(a.PW) + static_cast<uint32_t>(2 * xp)) * 8u;
    }
    u32x3 pr[NITMAX];
    // branch-free: a pair outside the image (the zero border) or a lane without a pair gets an offset past the
    // descriptor and reads zeros
    auto load_patch = [&](const Tile& t) __attribute__((always_inline)) {
        const int y0 = t.p0 * a.sh - a.ph, x0 = t.q0 * a.sw - a.pw - a.xoff;
        // 32-bit wrapping arithmetic: the offset of every pair that lies inside the image is in [0, x_bytes)
        const uint32_t base = ((static_cast<uint32_t>(t.img) * a.H + static_cast<uint32_t>(y0)) * a.W + static_cast<uint32_t>(x0)) * 6u;
#pragma unroll
        for (int it = 0; it < NITMAX; ++it) {
            const bool ok = (static_cast<unsigned>(y0 + py[it]) < static_cast<unsigned>(a.H)) &
                            (static_cast<unsigned>(x0 + px[it]) < static_cast<unsigned>(a.W));
            pr[it] = __builtin_bit_cast(u32x3, __builtin_amdgcn_raw_buffer_load_b96(rx, ok ? base + goff[it] : kBufOutside, 0, 0));
        }
    };
    // registers -> LDS, widened to four channels: [c0 c1 | c2 c0' | c1' c2'] -> [c0 c1 | c2 0 | c0' c1' | c2' 0]
    auto store_patch = [&](unsigned char* buf) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < NITMAX; ++it) {
            if (has[it]) {
                const u32x3 d = pr[it];
                const u32x4 w = {d[0], d[1] & 0xFFFFu, (d[1] >> 16) | (d[2] << 16), d[2] >> 16};
                *reinterpret_cast<u32x4*>(buf + loff[it]) = w;
            }
        }
    };

    // per-lane fragment base inside a patch: pixel (row block mi: rows wm*4 + mi*2 + (lrow >> 4), column lrow & 15)
    int pbase[2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
        pbase[mi] = (((wm * 4 + mi * 2 + (lrow >> 4)) * a.sh) * a.PW + (lrow & 15) * a.sw + 2 * lh) * 8;

    // byte offset of step ks inside a patch (filter row r, tap group h); 0 for the zero-weight steps past ktot
    int koff[KMAX];
    {
        int r = 0, h = 0;
#pragma unroll
        for (int ks = 0; ks < KMAX; ++ks) {
            koff[ks] = (ks < a.ktot) ? (r * a.PW + 4 * h) * 8 : 0;
            if (++h == a.kpr) {
                h = 0;
                ++r;
            }
        }
    }

    typedef short s16x2 __attribute__((ext_vector_type(2)));
    const s16x2 floor2 = __builtin_bit_cast(s16x2, a.relu ? 0u : 0x80008000u);
    f32x16 acc[2];
    unsigned char* stg = stg_base + wave * (64 * 80);
    // read-back lane (it): staged row it*16 + lane/4 = pixel row wm*4 + it (+ lane/64...), 16-byte chunk lane&3;
    // its byte offset in Y relative to the tile's first pixel and channel n0
    uint32_t yoff[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int row = it * 16 + (lane >> 2);
        yoff[it] = ((static_cast<uint32_t>(wm * 4 + (row >> 4)) * a.Q + static_cast<uint32_t>(row & 15)) * a.O +
                    static_cast<uint32_t>(wn * 32 + (lane & 3) * 8)) * 2u;
    }

    // Optional one-time start stagger by residency slot (TWN_FIRST_STAGGER, in units of 512 cycles; off by
    // default: measured without effect, the workgroups of a CU drift apart on their own)
    {
        const int slot = static_cast<int>((blockIdx.x >> 8) % 3u);
        for (int d = 0; d < slot * a.stagger; ++d) __builtin_amdgcn_s_sleep(8);
    }
    TWN_FTRACE(1);
    // Order per tile i: MFMA loop; wait for everything in flight; patch i+1 registers -> LDS; request patch i+2;
    // epilogue and output stores of tile i; barrier.  A patch request so has a whole tile's time to be answered
    // (the input comes from memory: with the request at the top of the tile that consumes it, a third of the
    // kernel's time was spent waiting for it), and it is older than the stores it would otherwise queue behind.
    Tile cur = tile_of(0);
    load_patch(cur);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    store_patch(smem);
    Tile nxt = cur;
    if (n_my > 1) {
        nxt = tile_of(1);
        load_patch(nxt);
    }
    // the first patch is in LDS (a bare barrier: the request just issued stays in flight)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    TWN_FTRACE(2);
    int buf = 0;
    for (uint32_t i = 0; i < n_my; ++i) {
        const bool more = (i + 1 < n_my), more2 = (i + 2 < n_my);
        const unsigned char* pb = smem + buf * a.patch_bytes;
        if (i == 1) TWN_FTRACE(3);
        {
            // All KMAX steps run (the weights of steps beyond ktot are zero and their fragments re-read offset 0):
            // straight-line code, so that the fragment reads of two groups of steps are in flight while a group
            // is multiplied (the compiler places exact lgkmcnt waits in straight-line code).
            constexpr int GRP = 2, NG = KMAX / GRP;
            static_assert(KMAX % GRP == 0, "steps per group");
            u32x4 af[3][GRP][2];
            auto load_group = [&](int g, u32x4 (*dst)[2]) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < GRP; ++u)
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi) {
                        const unsigned char* src = pb + pbase[mi] + koff[g * GRP + u];
                        if constexpr (EVEN_SW) {
                            dst[u][mi] = *reinterpret_cast<const u32x4*>(src);
                        } else {
                            // with an odd stride the fragment is only 8-byte aligned
                            const u32x2 lo = *reinterpret_cast<const u32x2*>(src);
                            const u32x2 hi = *reinterpret_cast<const u32x2*>(src + 8);
                            dst[u][mi] = u32x4{lo[0], lo[1], hi[0], hi[1]};
                        }
                    }
            };
            load_group(0, af[0]);
            if (NG > 1) load_group(1, af[1]);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                if (g + 2 < NG) load_group(g + 2, af[(g + 2) % 3]);
#pragma unroll
                for (int u = 0; u < GRP; ++u)
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi) {
                        // the first step starts from a zero C operand (an inline constant): no clearing pass
                        const f32x16 c_in = (g == 0 && u == 0) ? f32x16{} : acc[mi];
                        acc[mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfrag[g * GRP + u]),
                                                                          __builtin_bit_cast(bf16x8, af[g % 3][u][mi]),
                                                                          c_in, 0, 0, 0);
                    }
            }
        }
        if (i == 1) TWN_FTRACE(4);
        // a full wait, not a counted one: it does not rest on requests being answered in issue order when all lanes
        // of one fall outside the image; it covers the stores of tile i-1 too, which have had a tile's time
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (more) store_patch(smem + (buf ^ 1) * a.patch_bytes);
        Tile nn = nxt;
        if (more2) {
            nn = tile_of(i + 2);
            load_patch(nn);
        }
        if (i == 1) TWN_FTRACE(5);
        // ---- epilogue: accumulator element e of block mi in this lane: pixel row wm*4 + mi*2 + (lrow>>4),
        // column lrow & 15, channel wn*32 + (e>>2)*8 + lh*4 + (e&3) ----
        // both row blocks are staged before anything is read back: one LDS round trip per tile
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const int p = cur.p0 + wm * 4 + mi * 2 + (lrow >> 4), q = cur.q0 + (lrow & 15);
            const int64_t m = (static_cast<int64_t>(cur.img) * a.P + p) * a.Q + q;
            const bool pix_ok = p < a.P && q < a.Q;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int nl = wn * 32 + q4 * 8 + lh * 4;
                const f32x4 mul = *reinterpret_cast<const f32x4*>(colmul + nl);
                const f32x4 add = *reinterpret_cast<const f32x4*>(coladd + nl);
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[mi][q4 * 4 + e] * mul[e] + add[e];
                if (a.residual && pix_ok && n0 + nl < a.O) {
                    const u32x2 rr = *reinterpret_cast<const u32x2*>(a.residual + m * a.O + n0 + nl);
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
                *reinterpret_cast<u32x2*>(stg + (mi * 32 + lrow) * 80 + (q4 * 8 + lh * 4) * 2) = pk;
            }
        }
        // same wave wrote and reads: LDS executes a wave's operations in order
        {
            u32x4 val[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) val[it] = *reinterpret_cast<const u32x4*>(stg + (it * 16 + (lane >> 2)) * 80 + (lane & 3) * 16);
            // byte offset of the tile's first pixel and channel n0 (wave-uniform); a lane outside the tensor gets an offset
            // past the descriptor and its store is dropped
            const uint32_t ytile = (((static_cast<uint32_t>(cur.img) * a.P + static_cast<uint32_t>(cur.p0)) * a.Q +
                                     static_cast<uint32_t>(cur.q0)) * static_cast<uint32_t>(a.O) + static_cast<uint32_t>(n0)) * 2u;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int row = it * 16 + (lane >> 2);
                const bool ok = (cur.p0 + wm * 4 + (row >> 4) < a.P) & (cur.q0 + (row & 15) < a.Q) & (n0 + wn * 32 + (lane & 3) * 8 < a.O);
                const uint32_t vo = ok ? yoff[it] + ytile : kBufOutside;
                if (a.through) __builtin_amdgcn_raw_buffer_store_b128(val[it], ry, vo, 0, kStoreThrough);
                else __builtin_amdgcn_raw_buffer_store_b128(val[it], ry, vo, 0, 0);
            }
        }
        // The next patch is complete (this wave's LDS writes have landed) and every wave is done with the current
        // one.  A bare barrier: __syncthreads() would also wait for the epilogue's global stores, i.e. for a
        // write round trip to memory per tile.
        if (i == 1) TWN_FTRACE(6);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (i == 1) TWN_FTRACE(7);
        buf ^= 1;
        cur = nxt;
        nxt = nn;
    }
    TWN_FTRACE(8);
}

// ---- host side ------------------------------------------------------------------------------------------

static bool first_plan(const FirstLayer& f, FirstArgs* a) {
    if (f.C != 3 || f.R < 1 || f.R > 7 || f.S < 1 || f.S > 7 || f.sh < 1 || f.sw < 1 || f.sh > 2 || f.sw > 2) return false;
    if (f.W % 2 != 0 || f.O % 8 != 0) return false;
    if (!aligned(f.X, 4) || !aligned(f.Wq, 16) || !aligned(f.Y, 16) || (f.residual && !aligned(f.residual, 8))) return false;
    const int xoff = f.pw & 1;
    const int kpr = (f.S + xoff + 3) / 4, ktot = f.R * kpr;
    if (ktot > 14) return false;
    const int64_t xb = static_cast<int64_t>(f.N) * f.H * f.W * 6;
    if (xb >= (1LL << 31)) return false;
    const int64_t K = static_cast<int64_t>(f.R) * f.S * 3;
    if (twn_packed_words_per_row(K) > 16) return false;
    // the row builder reads three consecutive packed words from the first word of a filter row
    if ((((f.R - 1) * f.S * 3) >> 4) + 2 >= twn_packed_words_per_row(K)) return false;
    a->X = f.X; a->Wq = f.Wq; a->alpha = f.alpha; a->scale = f.scale; a->shift = f.shift; a->residual = f.residual; a->Y = f.Y;
    a->N = f.N; a->H = f.H; a->W = f.W; a->O = f.O; a->R = f.R; a->S = f.S; a->sh = f.sh; a->sw = f.sw;
    a->ph = f.ph; a->pw = f.pw; a->P = f.P; a->Q = f.Q;
    a->wpr = static_cast<int32_t>(twn_packed_words_per_row(K));
    a->rows_per_group = f.rows_per_group;
    a->relu = f.relu;
    a->xoff = xoff; a->kpr = kpr; a->ktot = ktot;
    a->PH = (kFirstTH - 1) * f.sh + f.R;
    a->PW = ((kFirstTW - 1) * f.sw + 4 * kpr + 1) & ~1;
    a->pairs = a->PW / 2;
    a->patch_bytes = static_cast<int32_t>(round_up(static_cast<size_t>(a->PH) * a->PW * 8, 16));
    a->nit = (a->PH * a->pairs + 255) / 256;
    if (a->nit > 4) return false;
    a->tiles_x = static_cast<uint32_t>((f.Q + kFirstTW - 1) / kFirstTW);
    a->tiles_y = static_cast<uint32_t>((f.P + kFirstTH - 1) / kFirstTH);
    const int64_t tiles = static_cast<int64_t>(f.N) * a->tiles_x * a->tiles_y;
    if (tiles <= 0 || tiles >= (1LL << 30)) return false;
    a->tiles = static_cast<uint32_t>(tiles);
    a->divTX = make_fastdiv_u(a->tiles_x);
    a->divTY = make_fastdiv_u(a->tiles_y);
    a->divPairs = make_fastdiv_u(static_cast<uint32_t>(a->pairs));
    a->divKq = make_fastdiv_u(static_cast<uint32_t>(ktot * 8));
    // the expanded weight table (64 channels x ktot*32 bytes) is built where the patches and staging rows go
    if (64 * ktot * 32 > 2 * a->patch_bytes + kFirstStg) return false;
    a->x_bytes = static_cast<uint32_t>(xb);
    const int64_t yb = static_cast<int64_t>(f.N) * f.P * f.Q * f.O * 2;
    if (yb >= (1LL << 31)) return false;
    a->y_bytes = static_cast<uint32_t>(yb);
    a->stagger = env_int("TWN_FIRST_STAGGER", 0);
    // Ordinary stores by default: written through, this kernel alone is faster (ResNet-18 stem 35.6 -> 33.7 us) but the
    // step it is part of slower (0.442 -> 0.450 ms, A/B on one box): its 103 MB of output then drain into the next launch.
    a->through = env_int("TWN_FIRST_THROUGH", 0) != 0 ? 1 : 0;
    return true;
}

bool conv_first_applicable(const FirstLayer& f) {
    FirstArgs a;
    return first_plan(f, &a);
}

template <int KMAX>
static int32_t launch_first(const FirstArgs& a, hipStream_t st) {
    // patch pairs per lane: 1, 2 or 4 (a plan with 3 runs the build for 4: the fourth request of a lane reads zeros)
    auto pick = [&](auto nit_tag) {
        constexpr int NIT = decltype(nit_tag)::value;
        return (a.sw % 2 == 0) ? conv_first_kernel<KMAX, NIT, true> : conv_first_kernel<KMAX, NIT, false>;
    };
    auto k = a.nit <= 1 ? pick(std::integral_constant<int, 1>{})
             : a.nit == 2 ? pick(std::integral_constant<int, 2>{}) : pick(std::integral_constant<int, 4>{});
    const int smem = 2 * a.patch_bytes + kFirstStg + 2 * 64 * 4 + 64 * a.wpr * 4;
    static std::once_flag once;
    static int cus = 256;
    std::call_once(once, [] {
        int dev = 0;
        hipDeviceProp_t p;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess && p.multiProcessorCount > 0)
            cus = p.multiProcessorCount;
    });
    if (smem > 64 * 1024) return TWN_ERR_UNSUPPORTED;
    const unsigned tiles_n = static_cast<unsigned>((a.O + 63) / 64);
    int per_cu = (160 * 1024) / smem;
    if (per_cu > 3) per_cu = 3;
    const int cap = env_int("TWN_FIRST_OCC", 0);
    if (cap > 0 && cap < per_cu) per_cu = cap;
    int64_t gx = static_cast<int64_t>(cus) * per_cu / tiles_n;
    if (gx < 8) gx = 8;
    if (gx > a.tiles) gx = a.tiles;
    k<<<dim3(static_cast<unsigned>(gx), tiles_n), dim3(256), smem, st>>>(a);
    return launch_status();
}

int32_t launch_conv_first(const FirstLayer& f, hipStream_t st) {
    FirstArgs a;
    if (!first_plan(f, &a)) return TWN_ERR_UNSUPPORTED;
    return a.ktot <= 4 ? launch_first<4>(a, st) : launch_first<14>(a, st);
}

}  // namespace twn
