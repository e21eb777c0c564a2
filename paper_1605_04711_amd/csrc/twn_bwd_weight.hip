// Weight gradient of the straight-through backward (Alg. 1 steps 9-10):
//   dW[o][c][r][s] = sum_{n,p,q} X[n, p*sh-ph+r*dh, q*sw-pw+s*dw, c] * dY[n,p,q,o]
// This is dL/dT; it involves neither alpha nor the codes and is handed to the
// float32 master weights unchanged (identity straight-through estimator).
//
// Dense bf16 x bf16 -> fp32 MFMA GEMM  D[o][j] = sum_pix dY[pix][o] * Xg[pix][j],
// j = (r*S+s)*C + c.  The reduction index (pixels) is the slow index of both
// NHWC operands, so MFMA fragments (8 consecutive pixels of one channel per
// lane) need a transpose.  Main kernel (weight_grad_patch_kernel, channel counts
// multiples of 8): both tiles go global -> LDS untransposed with direct 16-byte
// LDS loads, three slabs of 32 pixels deep, and fragments are fetched with the
// gfx950 transposing LDS read ds_read_tr16_b64 (a 16-lane group reads a 4 pixel
// x 16 channel block and each lane receives 4 consecutive pixels of its own
// channel); 16-byte chunks are XOR-swizzled by 2*(pixel & 3) so the four pixel
// rows of a block fall in different banks.  Fallback kernel (weight_grad_kernel,
// any channel count): tiles are transposed on their way into LDS: a thread loads
// the same 8 channels of two neighbouring pixels (2 x 16 bytes, coalesced
// across lanes along the channel axis), interleaves them into eight 32-bit
// words {pixel, pixel+1} and writes those to rows [channel][pixel].  MFMA
// fragments are then plain ds_read_b128 along the pixel axis.  The 16-byte
// chunk index of a row is XOR-swizzled with (row & 7) ^ ((row >> 3) & 7), which
// keeps both the transposing writes and the fragment reads at the minimum
// number of LDS bank passes.  The pixel range is split over blockIdx.y; partial
// tiles go to a workspace and are summed in a fixed order (deterministic).
#include <type_traits>

#include <mutex>

#include "twn_kernels.h"
#include "twn_mfma.h"

namespace twn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Exact unsigned division of numerators below 2^31 by a runtime constant.
struct FastDiv {
    uint32_t mul, shift, d, one;   // one = all ones when d == 1 (then mul = 0 and the quotient is n itself)
};

static FastDiv make_fastdiv(uint32_t d) {
    FastDiv f{0, 0, d, 0xFFFFFFFFu};
    if (d <= 1) return f;
    f.one = 0;
    uint32_t l = 0;
    while ((1u << l) < d) ++l;
    const uint32_t s = 31 + l;
    f.mul = static_cast<uint32_t>(((1ULL << s) + d - 1) / d);
    f.shift = s - 32;
    return f;
}

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv& f) {
    return (__umulhi(n, f.mul) >> f.shift) | (n & f.one);
}

struct WGArgs {
    WeightGrad w;
    FastDiv divPQ, divQ, divC, divS;
    FastDiv divSX, divSY;       // patch kernel: slab index -> (batch, row, column) patch coordinates
    WgPlan plan;
    int64_t pixels;
    int32_t J;
    int32_t slabs_per_split;
    int32_t xcd_map;            // patch kernel: renumber workgroups so that an XCD owns a contiguous run of (range, tile)
    // patch kernel, buffer-descriptor loads (both tensors below 2 GiB): sizes in bytes; `exact` = every patch
    // lies inside the output image (N, P, Q are multiples of the patch extents)
    uint32_t dy_bytes, x_bytes;
    int32_t exact;
};

#ifndef TWN_WG_STORE_AUX
#define TWN_WG_STORE_AUX kStoreThrough
#endif
constexpr int kWgTile = 128;

__device__ __forceinline__ int wg_swz(int row, int chunk) { return chunk ^ (row & 7) ^ ((row >> 3) & 7); }

template <bool VEC>
__global__ __launch_bounds__(256) void weight_grad_kernel(const WGArgs a) {
    __shared__ __attribute__((aligned(16))) uint16_t At[2][kWgTile * 64];   // [o][pix]
    __shared__ __attribute__((aligned(16))) uint16_t Bt[2][kWgTile * 64];   // [j][pix]

    const WeightGrad& w = a.w;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lh = lane >> 5;

    const int tiles_j = (a.J + kWgTile - 1) / kWgTile;
    const int o0 = static_cast<int>(blockIdx.x / tiles_j) * kWgTile;
    const int j0 = static_cast<int>(blockIdx.x % tiles_j) * kWgTile;
    const int split = blockIdx.y;
    const int64_t slab_begin = static_cast<int64_t>(split) * a.slabs_per_split;
    const int64_t total_slabs = (a.pixels + 63) / 64;
    int64_t slab_end = slab_begin + a.slabs_per_split;
    if (slab_end > total_slabs) slab_end = total_slabs;

    // staging tasks: chunk column cc (8 channels) and pixel pairs pp0, pp0+16
    const int cc = tid & 15;
    const int pp0 = tid >> 4;
    // fixed per thread: the tap and channel of this thread's 8 columns of Xg
    const int jj = j0 + cc * 8;
    int tr = 0, ts = 0, tc = 0;
    if (VEC) {
        const uint32_t rs = fdiv(jj, a.divC);
        tc = jj - rs * w.C;
        tr = fdiv(rs, a.divS);
        ts = rs - tr * w.S;
    }
    const int oo = o0 + cc * 8;

    u32x4 ra[2][2], rb[2][2];   // [task][pixel of the pair]

    auto load_x_elem = [&](int64_t pix, int j) -> uint32_t {
        if (pix >= a.pixels || j >= a.J) return 0;
        const uint32_t n = fdiv(static_cast<uint32_t>(pix), a.divPQ);
        const uint32_t rem = static_cast<uint32_t>(pix) - n * a.divPQ.d;
        const uint32_t p = fdiv(rem, a.divQ);
        const uint32_t q = rem - p * w.Q;
        const uint32_t rs = fdiv(j, a.divC);
        const int c = j - rs * w.C;
        const int r = fdiv(rs, a.divS);
        const int s = rs - r * w.S;
        const int ih = static_cast<int>(p) * w.sh - w.ph + r * w.dh;
        const int iw = static_cast<int>(q) * w.sw - w.pw + s * w.dw;
        if (static_cast<unsigned>(ih) >= static_cast<unsigned>(w.H) ||
            static_cast<unsigned>(iw) >= static_cast<unsigned>(w.W)) return 0;
        return w.X[((static_cast<int64_t>(n) * w.H + ih) * w.W + iw) * w.C + c];
    };

    auto load_slab = [&](int64_t slab) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int64_t pix = slab * 64 + (pp0 + 16 * t) * 2 + e;
                if (VEC) {
                    const bool pok = pix < a.pixels;
                    ra[t][e] = (pok && oo < w.O)
                                   ? *reinterpret_cast<const u32x4*>(w.dY + pix * w.O + oo)
                                   : u32x4{0, 0, 0, 0};
                    bool ok = pok && jj < a.J;
                    int64_t off = 0;
                    if (ok) {
                        const uint32_t n = fdiv(static_cast<uint32_t>(pix), a.divPQ);
                        const uint32_t rem = static_cast<uint32_t>(pix) - n * a.divPQ.d;
                        const uint32_t p = fdiv(rem, a.divQ);
                        const uint32_t q = rem - p * w.Q;
                        const int ih = static_cast<int>(p) * w.sh - w.ph + tr * w.dh;
                        const int iw = static_cast<int>(q) * w.sw - w.pw + ts * w.dw;
                        ok = static_cast<unsigned>(ih) < static_cast<unsigned>(w.H) &&
                             static_cast<unsigned>(iw) < static_cast<unsigned>(w.W);
                        off = ((static_cast<int64_t>(n) * w.H + ih) * w.W + iw) * w.C + tc;
                    }
                    rb[t][e] = ok ? *reinterpret_cast<const u32x4*>(w.X + off) : u32x4{0, 0, 0, 0};
                } else {
                    uint32_t va[4] = {0, 0, 0, 0}, vb[4] = {0, 0, 0, 0};
                    for (int i = 0; i < 8; ++i) {
                        uint32_t x = 0;
                        if (pix < a.pixels && oo + i < w.O) x = w.dY[pix * w.O + oo + i];
                        va[i >> 1] |= x << ((i & 1) * 16);
                        vb[i >> 1] |= load_x_elem(pix, jj + i) << ((i & 1) * 16);
                    }
                    ra[t][e] = u32x4{va[0], va[1], va[2], va[3]};
                    rb[t][e] = u32x4{vb[0], vb[1], vb[2], vb[3]};
                }
            }
        }
    };

    // interleave two pixels of 8 channels into 8 words {pix, pix+1} and write rows [channel][pixel]
    auto store_t = [&](uint16_t* dst, const u32x4& p0, const u32x4& p1, int pp) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t even = (p0[i] & 0xFFFFu) | (p1[i] << 16);
            const uint32_t odd = (p0[i] >> 16) | (p1[i] & 0xFFFF0000u);
            const int row0 = cc * 8 + 2 * i;
            const int chunk = pp >> 2;
            *reinterpret_cast<uint32_t*>(&dst[row0 * 64 + wg_swz(row0, chunk) * 8 + (pp & 3) * 2]) = even;
            *reinterpret_cast<uint32_t*>(&dst[(row0 + 1) * 64 + wg_swz(row0 + 1, chunk) * 8 + (pp & 3) * 2]) = odd;
        }
    };

    auto store_slab = [&](int buf) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            store_t(At[buf], ra[t][0], ra[t][1], pp0 + 16 * t);
            store_t(Bt[buf], rb[t][0], rb[t][1], pp0 + 16 * t);
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.0f;

    if (slab_begin < slab_end) {
        load_slab(slab_begin);
        store_slab(0);
    }
    __syncthreads();
    for (int64_t slab = slab_begin; slab < slab_end; ++slab) {
        const int cur = static_cast<int>((slab - slab_begin) & 1);
        const bool more = slab + 1 < slab_end;
        if (more) load_slab(slab + 1);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 af[2], bf[2];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const int row = wm * 64 + mi * 32 + lrow;
                af[mi] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const u32x4*>(&At[cur][row * 64 + wg_swz(row, lh * 4 + kk) * 8]));
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const int row = wn * 64 + ni * 32 + lrow;
                bf[ni] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const u32x4*>(&Bt[cur][row * 64 + wg_swz(row, lh * 4 + kk) * 8]));
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bf[ni], acc[mi][ni], 0, 0, 0);
        }
        if (more) store_slab(cur ^ 1);
        __syncthreads();
    }

    float* out = w.partial + static_cast<int64_t>(split) * w.O * a.J;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int j = j0 + wn * 64 + ni * 32 + lrow;
            if (j >= a.J) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int o = o0 + wm * 64 + mi * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
                if (o < w.O) out[static_cast<int64_t>(o) * a.J + j] = acc[mi][ni][e];
            }
        }
}

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __attribute__((aligned(16))) const uint32_t kWgZeroBlock[4] = {0u, 0u, 0u, 0u};

constexpr int wg_vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

__device__ __forceinline__ void wg_dma16(const void* gsrc, void* lds_dst) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                     (__attribute__((address_space(3))) void*)lds_dst, 16, 0, 0);
}

// Transposing LDS read of 4 pixels x 16 bits for this lane (see the file header).  Issued as inline
// assembly: the compiler would otherwise order every LDS read after ALL outstanding direct-to-LDS
// loads (s_waitcnt vmcnt(0)), which serialises the software pipeline.  The caller waits for the data
// with wg_wait<N>() + wg_ready() before using it.
template <int OFFSET>
__device__ __forceinline__ u32x2 wg_tr_read(uint32_t lds_addr) {
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(lds_addr), "n"(OFFSET));
    return v;
}

// s_waitcnt lgkmcnt(N): at most N of the LDS reads issued so far are still outstanding (they complete in
// issue order).  wg_ready ties the consumers of fragment registers to the preceding wait.
template <int N>
__device__ __forceinline__ void wg_wait() {
    static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N));
}
__device__ __forceinline__ void wg_ready(u32x2 (&f)[2][2]) {
    asm volatile("" : "+v"(f[0][0]), "+v"(f[0][1]), "+v"(f[1][0]), "+v"(f[1][1]));
}
__device__ __forceinline__ void wg_ready_b(u32x2 (&f)[2]) {
    asm volatile("" : "+v"(f[0]), "+v"(f[1]));
}

__device__ __forceinline__ bf16x8 wg_join(const u32x2& lo, const u32x2& hi) {
    const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(bf16x8, v);
}

// Patch variant: 128 (o) x 256 (j) tile, reduction slabs of 32 pixels that form a pn x ph x pw patch of
// the output images.  The sum over pixels is order-free, so enumerating them patch by patch instead of
// linearly costs nothing and makes addressing cheap: the patch origin is uniform per slab (scalar
// arithmetic), a lane's offsets inside the patch are fixed, and no per-lane division is left.
// Waves 2 (o) x 2 (j): wave tile 64 x 128; wave column wn owns one 128-column half of the B tile.
// BUF: loads go through buffer descriptors.  A lane's byte offsets inside a patch are fixed; the patch origin
// is wave-uniform (scalar arithmetic), and a lane whose pixel, tap or channel is outside gets an offset beyond
// the descriptor's size and reads zeros: no 64-bit address arithmetic and no branches are left in the loop.
// EXACT (buffer path only): every patch lies inside the output image, so no lane tests its output pixel.
// KS = 2: the workgroup holds two groups of four waves that work on the SAME tile; group kg takes the slabs
// kg, kg+2, ... of the workgroup's pixel range in its own pipeline stages, and the two accumulator tiles are
// summed through LDS (group 1 first, a fixed order) before group 0 writes.  One such workgroup per CU keeps the
// eight waves per CU of two four-wave workgroups but dumps half as many partial tiles.
// O64 (layers with at most 64 filters): the four waves of a group sit side by side along j (wave tile 64 x 64) and
// multiply only the lower 64 rows of the dY tile, instead of spending half of every MFMA on rows that do not exist.
template <int STAGES, bool BUF, bool EXACT, int KS, bool O64>
__global__ __launch_bounds__(256 * KS, 2) void weight_grad_patch_kernel(const WGArgs a) {
    constexpr int NI = O64 ? 2 : 4;                 // 32-column blocks of a wave's tile
    constexpr int A_BYTES = 32 * 256;               // 32 pixels x 128 channels bf16
    constexpr int B_BYTES = 2 * A_BYTES;            // two 128-column halves
    constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int PD = STAGES - 1;
    constexpr int PER_STAGE = 6;                    // direct LDS loads per wave per slab
    static_assert(KS == 1 || KS == 2, "pixel groups per workgroup");
    extern __shared__ __attribute__((aligned(1024))) unsigned char wsm_all[];

    const WeightGrad& w = a.w;
    const WgPlan& pl = a.plan;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = (KS == 1) ? 0 : (wave_all >> 2);     // pixel group
    const int wave = wave_all & 3;                      // wave inside the group
    unsigned char* wsm = wsm_all + kg * (STAGES * STAGE_BYTES);
    // LDS byte address of the group's stages (low 32 bits of the generic address are the LDS offset)
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) unsigned char*)wsm));
    const int wm = O64 ? 0 : (wave >> 1);           // 64-row block of the tile
    const int wh = O64 ? (wave >> 1) : (wave & 1);  // 128-column half of the B tile the wave reads
    const int wc = O64 ? (wave & 1) * 64 : 0;       // first column inside that half
    const int wcol = wh * 128 + wc;                 // first column of the wave's tile inside the 256-column tile
    const int lrow = lane & 31, lh = lane >> 5;

    // Workgroups are dealt round-robin to the 8 XCDs in dispatch order (x fastest).  The tiles of one pixel
    // range read the same dY and overlapping X: give each XCD a contiguous run of (range, tile) pairs, tile
    // fastest, so that those tiles run side by side under one L2 instead of on eight.
    uint32_t bx = blockIdx.x, by = blockIdx.y;
    if (a.xcd_map) {
        const uint32_t nbx = gridDim.x, nb = nbx * gridDim.y, lin = by * nbx + bx;
        const uint32_t q = nb >> 3, r = nb & 7, xcd = lin & 7, idx = lin >> 3;
        const uint32_t t = (xcd < r) ? xcd * (q + 1) + idx : r * (q + 1) + (xcd - r) * q + idx;
        bx = t % nbx;
        by = t / nbx;
    }
    const int tiles_j = (a.J + 255) / 256;
    const int o0 = static_cast<int>(bx / tiles_j) * 128;
    const int j0 = static_cast<int>(bx % tiles_j) * 256;
    const int64_t slab_begin = static_cast<int64_t>(by) * a.slabs_per_split;
    int64_t slab_end = slab_begin + a.slabs_per_split;
    if (slab_end > pl.slabs) slab_end = pl.slabs;
    const int nslab = static_cast<int>(slab_end - slab_begin);
    // group kg multiplies the slabs slab_begin + kg + KS*i; every group runs the same number of loop rounds
    // (the barriers are workgroup-wide), a round past the group's last slab loads zeros
    const int nround = (nslab + KS - 1) / KS;
    auto round_live = [&](int i) __attribute__((always_inline)) -> bool { return i * KS + kg < nslab; };
    const void* zero = kWgZeroBlock;

    // ---- loader: a wave-level load covers 4 pixel rows x 256 bytes; this wave loads row groups wave and wave+4 ----
    const int prow = lane >> 4;
    const int qch = (lane & 15) ^ (2 * (prow & 3));     // logical 8-channel chunk fetched by this lane
    const int oo = o0 + qch * 8;
    const bool ook = oo < w.O;
    int tc[2], th0[2], tw0[2];
    bool jok[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int jj = j0 + h * 128 + qch * 8;
        const uint32_t rs = fdiv(jj, a.divC);
        tc[h] = jj - static_cast<int>(rs) * w.C;
        const int tr = static_cast<int>(fdiv(rs, a.divS));
        const int ts = static_cast<int>(rs) - tr * w.S;
        th0[h] = tr * w.dh - w.ph;
        tw0[h] = ts * w.dw - w.pw;
        jok[h] = jj < a.J;
    }
    // offsets of this lane's two pixels inside a patch (local pixel l = 4*group + prow)
    const int lpw = __builtin_ctz(pl.pw), lph = __builtin_ctz(pl.ph);
    int dn[2], dy[2], dx[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int l = 4 * (wave + 4 * t) + prow;
        dx[t] = l & (pl.pw - 1);
        dy[t] = (l >> lpw) & (pl.ph - 1);
        dn[t] = l >> (lpw + lph);
    }

    // buffer path: fixed per-lane byte offsets relative to the patch origin
    const __amdgpu_buffer_rsrc_t rdy = make_rsrc(w.dY, a.dy_bytes), rx = make_rsrc(w.X, a.x_bytes);
    uint32_t voffA[2] = {0u, 0u};
    uint32_t voffB[2][2] = {{0u, 0u}, {0u, 0u}};      // may stand for a negative offset (arithmetic is modulo 2^32)
    int32_t aH[2][2], aW[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        if constexpr (BUF) {
            const uint32_t pix = (static_cast<uint32_t>(dn[t]) * w.P + dy[t]) * w.Q + dx[t];
            voffA[t] = ook ? (pix * w.O + oo) * 2u : kBufOutside;
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            aH[t][h] = dy[t] * w.sh + th0[h];
            aW[t][h] = dx[t] * w.sw + tw0[h];
            if constexpr (BUF) {
                // a column beyond J never passes the row test below (no separate test per load)
                if (!jok[h]) aH[t][h] = 0x40000000;
                const uint32_t pix = (static_cast<uint32_t>(dn[t]) * w.H + static_cast<uint32_t>(aH[t][h])) * w.W +
                                     static_cast<uint32_t>(aW[t][h]);
                voffB[t][h] = (pix * w.xc + tc[h]) * 2u;
            }
        }
    }

    // buffer path: the calls of issue() walk consecutive slabs, so the patch coordinates (cx, cy, cn) are kept
    // as running scalar counters and every uniform offset is three multiplications by a per-launch stride
    uint32_t cx, cy, cn;
    {
        const uint32_t su = static_cast<uint32_t>(slab_begin) + static_cast<uint32_t>(kg);
        const uint32_t t1 = fdiv(su, a.divSX);
        cx = su - t1 * pl.sx;
        cn = fdiv(t1, a.divSY);
        cy = t1 - cn * pl.sy;
    }
    const uint32_t strAx = static_cast<uint32_t>(pl.pw) * w.O * 2u, strAy = static_cast<uint32_t>(pl.ph) * w.Q * w.O * 2u,
                   strAn = static_cast<uint32_t>(pl.pn) * w.P * w.Q * w.O * 2u;
    const uint32_t strBx = static_cast<uint32_t>(pl.pw) * w.sw * w.xc * 2u,
                   strBy = static_cast<uint32_t>(pl.ph) * w.sh * w.W * w.xc * 2u,
                   strBn = static_cast<uint32_t>(pl.pn) * w.H * w.W * w.xc * 2u;
    const int strH = pl.ph * w.sh, strW = pl.pw * w.sw;

    auto issue = [&](int64_t slab, int stage, bool live) __attribute__((always_inline)) {
        unsigned char* sA = wsm + stage * STAGE_BYTES;
        unsigned char* sB = sA + A_BYTES;
        if constexpr (BUF) {
            // a slab past the end of the range (live == false) still issues its loads, all of them reading zeros
            const uint32_t sA_off = live ? cn * strAn + cy * strAy + cx * strAx : 0u;
            const uint32_t sB_off = cn * strBn + cy * strBy + cx * strBx;
            const int hb = static_cast<int>(cy) * strH, wb = static_cast<int>(cx) * strW;
            const int remN = w.N - static_cast<int>(cn) * pl.pn, remP = w.P - static_cast<int>(cy) * pl.ph,
                      remQ = w.Q - static_cast<int>(cx) * pl.pw;      // unused when EXACT
            // advance to the patch of this group's next slab
#pragma unroll
            for (int adv = 0; adv < KS; ++adv) {
                ++cx;
                if (cx == static_cast<uint32_t>(pl.sx)) {
                    cx = 0;
                    ++cy;
                    if (cy == static_cast<uint32_t>(pl.sy)) {
                        cy = 0;
                        ++cn;
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                // bitwise, not short-circuit: straight-line code (selects), no branches around the loads
                const bool pok = EXACT ? live : (live & (dn[t] < remN) & (dy[t] < remP) & (dx[t] < remQ));
                buf_dma16(rdy, pok ? voffA[t] : kBufOutside, sA_off, sA + (wave + 4 * t) * 1024);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const bool bok = pok & (static_cast<unsigned>(hb + aH[t][h]) < static_cast<unsigned>(w.H)) &
                                     (static_cast<unsigned>(wb + aW[t][h]) < static_cast<unsigned>(w.W));
                    buf_dma16(rx, bok ? voffB[t][h] + sB_off : kBufOutside, 0u,
                              sB + h * A_BYTES + (wave + 4 * t) * 1024);
                }
            }
            return;
        }
        // patch origin: uniform over the workgroup
        const uint32_t su = static_cast<uint32_t>(slab);
        const uint32_t t1 = fdiv(su, a.divSX);
        const uint32_t sx = su - t1 * pl.sx;
        const uint32_t sn = fdiv(t1, a.divSY);
        const uint32_t sy = t1 - sn * pl.sy;
        const int n0 = static_cast<int>(sn) * pl.pn, p0 = static_cast<int>(sy) * pl.ph, q0 = static_cast<int>(sx) * pl.pw;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int n = n0 + dn[t], p = p0 + dy[t], q = q0 + dx[t];
            const bool pok = live && n < w.N && p < w.P && q < w.Q;
            const uint32_t opix = (static_cast<uint32_t>(n) * w.P + p) * w.Q + q;
            const void* srcA = (pok && ook) ? static_cast<const void*>(w.dY + static_cast<uint64_t>(opix) * w.O + oo)
                                            : zero;
            wg_dma16(srcA, sA + (wave + 4 * t) * 1024);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int ih = p * w.sh + th0[h], iw = q * w.sw + tw0[h];
                const bool bok = pok && jok[h] && static_cast<unsigned>(ih) < static_cast<unsigned>(w.H) &&
                                 static_cast<unsigned>(iw) < static_cast<unsigned>(w.W);
                const uint32_t ipix = (static_cast<uint32_t>(n) * w.H + ih) * w.W + iw;
                const void* srcB = bok ? static_cast<const void*>(w.X + static_cast<uint64_t>(ipix) * w.xc + tc[h])
                                       : zero;
                wg_dma16(srcB, sB + h * A_BYTES + (wave + 4 * t) * 1024);
            }
        }
    };

    // ---- fragment addressing (transposing read), as in the linear kernel ----
    const int li = lane & 15;
    const int fpix = 8 * lh + (li >> 2);
    const int fch = 16 * ((lane >> 4) & 1) + 4 * (li & 3);
    auto frag_off = [&](int chan0, int pixel) -> int {
        const int ch = chan0 + fch;
        const int chunk = (ch >> 3) ^ (2 * (pixel & 3));
        return pixel * 256 + chunk * 16 + (ch & 7) * 2;
    };
    int offA[2][2], offB[NI][2];
#pragma unroll
    for (int hv = 0; hv < 2; ++hv) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) offA[mi][hv] = frag_off(wm * 64 + mi * 32, fpix + 4 * hv);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) offB[ni][hv] = wh * A_BYTES + frag_off(wc + ni * 32, fpix + 4 * hv);
    }

    f32x16 acc[2][NI];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.0f;

    // ---- software pipeline ---------------------------------------------------------------------
    // A slab is two MFMA steps of eight MFMAs, taken as four pairs (mi = 0, 1) per channel tile ni.  The
    // fragments of the NEXT step are fetched while this one multiplies: the four dY fragments into the
    // other register set right after the first pair, the two halves of X fragment ni as soon as pair ni
    // has consumed the old ones.  LDS reads complete in issue order, so s_waitcnt lgkmcnt(n) with the
    // number of younger reads is exact: before the first pair of a step the 2*(NI-1) reads of the later X
    // fragments, before pair ni > 0 those plus what this step has issued so far, 2*NI + 2 in all.
    // Hand-over between the steps of slab `it`: slab it+1 has landed (its step 0 is prefetched during step
    // 1), and the stage of slab it-1, whose reads were all issued during step 0 of that slab, is refilled.
    u32x2 fa[2][2][2], fb[NI][2];
    // LDS byte addresses of this lane's fragments in stage 0; the stage and the half of the slab go into the
    // instruction's immediate offset (the loop is unrolled over the three stages), so a read costs no vector
    // arithmetic
    static_assert(STAGES == 3 && 2 * STAGE_BYTES + A_BYTES + 4096 < 65536, "immediate offsets of the fragment reads");
    uint32_t adrA[2][2], adrB[NI][2];
#pragma unroll
    for (int hv = 0; hv < 2; ++hv) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) adrA[mi][hv] = lds_base + offA[mi][hv];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) adrB[ni][hv] = lds_base + offB[ni][hv];
    }
    auto read_fa = [&](auto off_tag, u32x2 (*dst)[2]) __attribute__((always_inline)) {
        constexpr int OFF = decltype(off_tag)::value;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int hv = 0; hv < 2; ++hv) dst[mi][hv] = wg_tr_read<OFF>(adrA[mi][hv]);
    };
    auto read_fb = [&](auto off_tag, int ni) __attribute__((always_inline)) {
        constexpr int OFF = decltype(off_tag)::value + A_BYTES;
#pragma unroll
        for (int hv = 0; hv < 2; ++hv) fb[ni][hv] = wg_tr_read<OFF>(adrB[ni][hv]);
    };

#pragma unroll
    for (int s = 0; s < PD; ++s) issue(slab_begin + s * KS + kg, s, round_live(s));
    __builtin_amdgcn_s_waitcnt(wg_vmcnt_imm((PD - 1) * PER_STAGE));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    read_fa(std::integral_constant<int, 0>{}, fa[0]);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) read_fb(std::integral_constant<int, 0>{}, ni);

    // one slab that lives in stage STG (compile-time: the loop below walks the stages in order)
    auto slab = [&](int it, auto stg_tag) __attribute__((always_inline)) {
        constexpr int STG = decltype(stg_tag)::value;
        constexpr int NEXT = (STG + 1) % STAGES, FILL = (STG + PD) % STAGES;
        auto step = [&](auto kk_tag) __attribute__((always_inline)) {
            constexpr int KK = decltype(kk_tag)::value;
            // where the next step's fragments live: second half of this slab, or first half of the next one
            using NOff = std::integral_constant<int, (KK == 0) ? STG * STAGE_BYTES + 4096 : NEXT * STAGE_BYTES>;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                if (ni == 0) wg_wait<2 * (NI - 1)>(); else wg_wait<2 * NI + 2>();
                if (ni == 0) wg_ready(fa[KK]);
                wg_ready_b(fb[ni]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg_join(fa[KK][mi][0], fa[KK][mi][1]),
                                                                          wg_join(fb[ni][0], fb[ni][1]), acc[mi][ni],
                                                                          0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (ni == 0) read_fa(NOff{}, fa[KK ^ 1]);
                read_fb(NOff{}, ni);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        step(std::integral_constant<int, 0>{});
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(wg_vmcnt_imm((PD - 2) * PER_STAGE));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue(slab_begin + (it + PD) * KS + kg, FILL, round_live(it + PD));
        __builtin_amdgcn_sched_barrier(0);
        step(std::integral_constant<int, 1>{});
    };
    for (int it = 0; it < nround; it += 3) {
        slab(it, std::integral_constant<int, 0>{});
        if (it + 1 < nround) slab(it + 1, std::integral_constant<int, 1>{});
        if (it + 2 < nround) slab(it + 2, std::integral_constant<int, 2>{});
    }
    // the fragments fetched ahead for the slab after the last one are never used: let them land, and drain
    // the trailing zero loads, before registers and LDS are reused
    wg_wait<0>();
    wg_ready(fa[0]);
    wg_ready(fa[1]);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) wg_ready_b(fb[ni]);
    __builtin_amdgcn_s_waitcnt(wg_vmcnt_imm(0));

    if constexpr (KS == 2) {
        // group 1 hands its accumulator tile to group 0 through LDS, one 32-row block (64 KB) at a time; every
        // wave of the workgroup passes all four barriers
        f32x4* red = reinterpret_cast<f32x4*>(wsm_all);
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            __syncthreads();        // the stages are free (first round: all loads landed, all fragments read)
            if (kg == 1) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const f32x16& t = acc[mi][ni];
                        red[((wave * 4 + ni) * 4 + q4) * 64 + lane] = f32x4{t[q4 * 4], t[q4 * 4 + 1], t[q4 * 4 + 2], t[q4 * 4 + 3]};
                    }
            }
            __syncthreads();
            if (kg == 0) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const f32x4 v = red[((wave * 4 + ni) * 4 + q4) * 64 + lane];
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[mi][ni][q4 * 4 + e] += v[e];
                    }
            }
        }
        if (kg != 0) return;        // after the last barrier
    }

    if (pl.splits == 1 && !w.pad_sp) {
        // the only range: write the gradient itself, [O][C][R][S], without a reduction pass
        const int RS = w.R * w.S;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int j = j0 + wcol + ni * 32 + lrow;
            if (j >= a.J) continue;
            const uint32_t rs = fdiv(j, a.divC);
            const int c = j - static_cast<int>(rs) * w.C;
            const int64_t col = static_cast<int64_t>(c) * RS + rs;
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int o = o0 + wm * 64 + mi * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
                    if (o >= w.O) continue;
                    float* dst = w.dW + static_cast<int64_t>(o) * a.J + col;
                    *dst = (w.beta != 0.0f) ? w.beta * *dst + acc[mi][ni][e] : acc[mi][ni][e];
                }
        }
        return;
    }
    // The partial tile is written through (see kStoreThrough): the reduction pass reads it right after this kernel,
    // and left dirty in L2 it would all be written back in one burst when the kernel ends.  One split's tile set is
    // far below 2 GiB (checked by the launcher), so offsets are 32-bit.
    float* out = w.partial + static_cast<int64_t>(by) * w.O * a.J;
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(out, 0x7FFFFFFFu);
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int j = j0 + wcol + ni * 32 + lrow;
            if (j >= a.J) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int o = o0 + wm * 64 + mi * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
                if (o < w.O)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[mi][ni][e]), rout,
                                                          static_cast<uint32_t>(o * a.J + j) * 4u, 0, TWN_WG_STORE_AUX);
            }
        }
}

// dW[o][c][r][s] = beta*dW + sum over splits (fixed order) of partial[split][o][(r*S+s)*C + c]
// `pad_sp` = 0: partial tiles are [O][(r*S+s)*C + c].  First-layer mode (`pad_sp` = Sp > 0): tiles are
// [O][(r*Sp+s)*4 + c] and entries with s >= S or c >= C are phantom (dropped).
// A block covers 64*VEC consecutive partial elements (one float4 or one float per lane); its four waves
// each sum every fourth split with several loads in flight, and the four sums are combined in a fixed
// order; the small output is scattered.  VEC = 4 needs the tile size O*J to be a multiple of 4.
template <int VEC>
__global__ __launch_bounds__(256) void weight_grad_reduce_kernel(const float* __restrict__ partial, int splits,
                                                                 int O, int C, int R, int S, int pad_sp, float beta,
                                                                 float* __restrict__ dW) {
    __shared__ float red[4][64 * VEC];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t id0 = (static_cast<int64_t>(blockIdx.x) * 64 + lane) * VEC;
    const int64_t Jsrc = pad_sp ? static_cast<int64_t>(R) * pad_sp * 4 : static_cast<int64_t>(R) * S * C;
    const int64_t total = Jsrc * O;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.0f;
    if (id0 < total) {
#pragma unroll 8
        for (int sp = wave; sp < splits; sp += 4) {
            const float* src = partial + static_cast<int64_t>(sp) * total + id0;
            if (VEC == 4) {
                const float4 t = *reinterpret_cast<const float4*>(src);
                acc[0] += t.x; acc[1 % VEC] += t.y; acc[2 % VEC] += t.z; acc[3 % VEC] += t.w;
            } else {
                acc[0] += src[0];
            }
        }
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) red[wave][lane * VEC + v] = acc[v];
    __syncthreads();
    // one element per thread: element `el` of the block's 64*VEC (VEC = 1: the first wave only)
    const int el = threadIdx.x;
    if (el >= 64 * VEC) return;
    const int64_t id = static_cast<int64_t>(blockIdx.x) * 64 * VEC + el;
    if (id >= total) return;
    const float sum = ((red[0][el] + red[1][el]) + red[2][el]) + red[3][el];
    const int64_t o = id / Jsrc;
    const int64_t j = id - o * Jsrc;
    int64_t rs, c;
    int r, sx;
    if (pad_sp) {
        c = j & 3;
        rs = j >> 2;
        r = static_cast<int>(rs / pad_sp);
        sx = static_cast<int>(rs - static_cast<int64_t>(r) * pad_sp);
        if (c >= C || sx >= S) return;
    } else {
        rs = j / C;                  // = r*S + s
        c = j - rs * C;
        r = static_cast<int>(rs / S);
        sx = static_cast<int>(rs - static_cast<int64_t>(r) * S);
    }
    const int64_t dst = ((o * C + c) * R + r) * S + sx;   // [O][C][R][S]
    dW[dst] = (beta != 0.0f) ? beta * dW[dst] + sum : sum;
}

// The same reduction for few splits and many outputs (C % 64 == 0, no first-layer padding).  The kernel
// above scatters its sums as single floats, R*S floats apart; with few splits that write pattern is most of
// its time.  Here a block owns filter o and 64 consecutive channels: per tap it reads one 256-byte run of
// every split (float4 per lane, several splits in flight, summed in split order), transposes the R*S x 64
// sums through LDS and writes dW[o][c0..c0+63][:][:] as ONE contiguous run of 64*R*S floats.
constexpr int kReduceRowsMaxTaps = 25;
__global__ __launch_bounds__(256) void weight_grad_reduce_rows_kernel(const float* __restrict__ partial, int splits,
                                                                      int O, int C, int RS, float beta,
                                                                      float* __restrict__ dW) {
    __shared__ float tile[64 * kReduceRowsMaxTaps];      // [channel][tap]
    const int cchunks = C / 64;
    const int o = blockIdx.x / cchunks, c0 = (blockIdx.x % cchunks) * 64;
    const int64_t J = static_cast<int64_t>(RS) * C;
    const int64_t total = J * O;
    // item = (tap, group of 4 channels): 16 items per tap
    for (int item = threadIdx.x; item < RS * 16; item += 256) {
        const int rs = item >> 4, c4 = (item & 15) * 4;
        const float* src = partial + static_cast<int64_t>(o) * J + static_cast<int64_t>(rs) * C + c0 + c4;
        float4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 8
        for (int sp = 0; sp < splits; ++sp) {
            const float4 t = *reinterpret_cast<const float4*>(src + static_cast<int64_t>(sp) * total);
            acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
        }
        tile[(c4 + 0) * RS + rs] = acc.x;
        tile[(c4 + 1) * RS + rs] = acc.y;
        tile[(c4 + 2) * RS + rs] = acc.z;
        tile[(c4 + 3) * RS + rs] = acc.w;
    }
    __syncthreads();
    float* dst = dW + (static_cast<int64_t>(o) * C + c0) * RS;      // [O][C][R][S]: 64*RS contiguous floats
    for (int i = threadIdx.x; i < 64 * RS; i += 256) dst[i] = (beta != 0.0f) ? beta * dst[i] + tile[i] : tile[i];
}

// dbias partials: block (x = 64-channel group, y = pixel split) sums its pixel range.
constexpr int kBiasSplits = 64;
__global__ __launch_bounds__(256) void bias_grad_partial_kernel(const uint16_t* __restrict__ dY, int64_t pixels,
                                                                int O, float* __restrict__ partial) {
    __shared__ float red[4][64];
    const int ch = blockIdx.x * 64 + (threadIdx.x & 63);
    const int py = threadIdx.x >> 6;
    const int64_t per = (pixels + kBiasSplits - 1) / kBiasSplits;
    const int64_t begin = blockIdx.y * per;
    int64_t end = begin + per;
    if (end > pixels) end = pixels;
    float s = 0.0f;
    if (ch < O)
        for (int64_t p = begin + py; p < end; p += 4) s += bf16_to_f32(dY[p * O + ch]);
    red[py][threadIdx.x & 63] = s;
    __syncthreads();
    if (py == 0 && ch < O) partial[static_cast<int64_t>(blockIdx.y) * O + ch] = ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
}

__global__ __launch_bounds__(256) void bias_grad_final_kernel(const float* __restrict__ partial, int O,
                                                              float* __restrict__ dbias) {
    const int ch = blockIdx.x * blockDim.x + threadIdx.x;
    if (ch >= O) return;
    float s = 0.0f;
    for (int i = 0; i < kBiasSplits; ++i) s += partial[static_cast<int64_t>(i) * O + ch];
    dbias[ch] = s;
}

static int32_t choose_splits(int64_t tiles, int64_t slabs, int ks = 1) {
    int64_t want = env_int("TWN_WG_BLOCKS", 512) / ks;
    // tiles x splits must not exceed the workgroups that are resident at once (two of four waves or one of eight
    // per CU), or the launch grows a second, nearly empty round
    int64_t splits = (tiles >= 256) ? 1 : want / tiles;
    if (splits > slabs) splits = slabs;
    if (splits > 256) splits = 256;
    if (splits < 1) splits = 1;
    // every split must own at least one slab
    const int64_t per = (slabs + splits - 1) / splits;
    return static_cast<int32_t>((slabs + per - 1) / per);
}

WgPlan plan_weight_grad(int32_t N, int32_t P, int32_t Q, int32_t C, int32_t O, int32_t R, int32_t S) {
    WgPlan pl{};
    const int64_t J = static_cast<int64_t>(R) * S * C;
    const int64_t pixels = static_cast<int64_t>(N) * P * Q;
    pl.patch = (C % 8 == 0) && (O % 8 == 0);
    if (!pl.patch) {
        pl.tiles = static_cast<int32_t>(((O + kWgTile - 1) / kWgTile) * ((J + kWgTile - 1) / kWgTile));
        pl.slabs = (pixels + 63) / 64;
        pl.splits = choose_splits(pl.tiles, pl.slabs);
        pl.ks = 1;
        return pl;
    }
    // 32-pixel patch pn x ph x pw (powers of two) that wastes the fewest padded pixels; ties go to wide rows
    int64_t best = -1;
    for (int lw = 5; lw >= 0; --lw)
        for (int lh = 5 - lw; lh >= 0; --lh) {
            const int pw = 1 << lw, ph = 1 << lh, pn = 32 / (pw * ph);
            const int64_t sx = (Q + pw - 1) / pw, sy = (P + ph - 1) / ph, sn = (N + pn - 1) / pn;
            const int64_t padded = sx * sy * sn;
            if (best < 0 || padded < best) {
                best = padded;
                pl.pn = pn; pl.ph = ph; pl.pw = pw;
                pl.sn = static_cast<int32_t>(sn); pl.sy = static_cast<int32_t>(sy); pl.sx = static_cast<int32_t>(sx);
            }
        }
    pl.slabs = best;
    pl.tiles = static_cast<int32_t>(((O + 127) / 128) * ((J + 255) / 256));
    // Layers with fewer tiles than CUs split the pixels over workgroups, and every workgroup dumps a partial tile
    // (128 KB) that the reduction pass reads back: two groups of waves per workgroup halve that traffic at the
    // same number of waves per CU.  TWN_WG_KS=1 keeps four-wave workgroups.
    pl.ks = (pl.tiles < 256 && env_int("TWN_WG_KS", 2) == 2 && pl.slabs >= 4) ? 2 : 1;
    pl.splits = choose_splits(pl.tiles, pl.slabs, pl.ks);
    return pl;
}

// One build of the patch kernel: the dynamic-LDS limit is raised once per build.
template <bool BUF, bool EXACT, int KS, bool O64>
static int32_t launch_patch(const WGArgs& a, dim3 grid, hipStream_t st) {
    constexpr int kStages = 3;
    constexpr int kSmem = KS * kStages * 3 * 32 * 256;
    auto k = weight_grad_patch_kernel<kStages, BUF, EXACT, KS, O64>;
    static std::once_flag once;
    static bool allowed = false;
    std::call_once(once, [&] {
        allowed = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, kSmem) ==
                  hipSuccess;
    });
    if (!allowed) return TWN_ERR_HIP;
    k<<<grid, 256 * KS, kSmem, st>>>(a);
    return TWN_OK;
}

int32_t launch_weight_grad(const WeightGrad& w, hipStream_t st) {
    WGArgs a;
    a.w = w;
    a.pixels = static_cast<int64_t>(w.N) * w.P * w.Q;
    a.J = w.R * w.S * w.C;
    a.divPQ = make_fastdiv(static_cast<uint32_t>(w.P) * w.Q);
    a.divQ = make_fastdiv(w.Q);
    a.divC = make_fastdiv(w.C);
    a.divS = make_fastdiv(w.S);
    if (a.pixels >= (1LL << 31)) return TWN_ERR_SHAPE;
    if (static_cast<int64_t>(w.O) * a.J >= (1LL << 28)) return TWN_ERR_SHAPE;   // 32-bit byte offsets inside one partial tile set
    a.plan = plan_weight_grad(w.N, w.P, w.Q, w.C, w.O, w.R, w.S);
    a.divSX = make_fastdiv(a.plan.patch ? a.plan.sx : 1);
    a.divSY = make_fastdiv(a.plan.patch ? a.plan.sy : 1);
    const int32_t splits = a.plan.splits;
    a.slabs_per_split = static_cast<int32_t>((a.plan.slabs + splits - 1) / splits);
    a.xcd_map = env_int("TWN_WG_XCD", 1);
    a.dy_bytes = a.x_bytes = 0;
    a.exact = 0;
    if (w.dW) {
        const dim3 grid(a.plan.tiles, splits);
        if (a.plan.patch) {
            const int64_t dyb = a.pixels * w.O * 2;
            const int64_t xb = ((static_cast<int64_t>(w.N) * w.H * w.W - 1) * w.xc + w.C) * 2;
            const bool buf = env_int("TWN_BUFLOAD", 1) != 0 && dyb < (1LL << 31) && xb < (1LL << 31);
            a.dy_bytes = static_cast<uint32_t>(buf ? dyb : 0);
            a.x_bytes = static_cast<uint32_t>(buf ? xb : 0);
            a.exact = (w.N % a.plan.pn == 0 && w.P % a.plan.ph == 0 && w.Q % a.plan.pw == 0) ? 1 : 0;
            const bool o64 = w.O <= 64;
            int32_t rc;
            auto pick = [&](auto buf_tag, auto exact_tag) {
                constexpr bool B = decltype(buf_tag)::value, E = decltype(exact_tag)::value;
                if (a.plan.ks == 2)
                    return o64 ? launch_patch<B, E, 2, true>(a, grid, st) : launch_patch<B, E, 2, false>(a, grid, st);
                return o64 ? launch_patch<B, E, 1, true>(a, grid, st) : launch_patch<B, E, 1, false>(a, grid, st);
            };
            if (buf && a.exact)
                rc = pick(std::true_type{}, std::true_type{});
            else if (buf)
                rc = pick(std::true_type{}, std::false_type{});
            else
                rc = pick(std::false_type{}, std::false_type{});
            if (rc != TWN_OK) return rc;
        } else {
            weight_grad_kernel<false><<<grid, 256, 0, st>>>(a);
        }
        if (w.pad_sp || !(a.plan.patch && splits == 1)) {   // a single-range patch launch writes dW itself
            const int64_t total = static_cast<int64_t>(w.O) * a.J;
            const int C = w.pad_sp ? w.c_real : w.C, S = w.pad_sp ? w.s_real : w.S;
            const int RS = w.R * w.S;
            if (!w.pad_sp && w.C % 64 == 0 && RS <= kReduceRowsMaxTaps && splits <= env_int("TWN_WG_ROWS_SPLITS", 32))
                weight_grad_reduce_rows_kernel<<<static_cast<unsigned>(w.O * (w.C / 64)), 256, 0, st>>>(
                    w.partial, splits, w.O, w.C, RS, w.beta, w.dW);
            else if (total % 4 == 0)
                weight_grad_reduce_kernel<4><<<static_cast<unsigned>((total + 255) / 256), 256, 0, st>>>(
                    w.partial, splits, w.O, C, w.R, S, w.pad_sp, w.beta, w.dW);
            else
                weight_grad_reduce_kernel<1><<<static_cast<unsigned>((total + 63) / 64), 256, 0, st>>>(
                    w.partial, splits, w.O, C, w.R, S, w.pad_sp, w.beta, w.dW);
        }
    }
    if (w.dbias) {
        float* bp = w.partial + static_cast<int64_t>(splits) * w.O * a.J;
        bias_grad_partial_kernel<<<dim3((w.O + 63) / 64, kBiasSplits), 256, 0, st>>>(w.dY, a.pixels, w.O, bp);
        bias_grad_final_kernel<<<(w.O + 255) / 256, 256, 0, st>>>(bp, w.O, w.dbias);
    }
    return launch_status();
}

}  // namespace twn
