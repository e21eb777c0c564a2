// Threshold ternarization on gfx950 (Sec. 2.3: rule of thumb for Delta, Eq. 3
// codes, Eq. 5 alpha; Alg. 1 steps 3-7).  HBM-streaming kernels:
//
//   abs_sum           pass 1: per-block float64 partial sums of |W|
//   mask_pack_flat    pass 2: Delta from the partials, then one more stream of W:
//                     masked float64 sum, count, and the 2-bit codes written in
//                     the same pass (flat layouts: R*S == 1 and K % 128 == 0)
//   mask_pack_gather  pass 2 for any [rows][C][R][S] layout: one thread per output
//                     word of the normal and of the transposed copy; the normal
//                     words also carry the masked sum and count
//   pack_gather       codes only (transposed copy of flat layouts, per-filter groups)
//   group_stats       one block per group when there are several groups (per filter)
//
//   finalize          fixed-order sum of the pass-2 partials -> Delta, alpha, nnz
//
// (A "last block finishes" variant with a ticket counter was measured and dropped:
// the device-scope release it needs writes back the L2 of every XCD once per block
// and cost 75 us on the 2^28 tensor.)  All floating-point sums run in a fixed
// order: results are bit-identical from run to run; no floating-point atomics.
#include <mutex>

#include "twn_common.h"

namespace twn {

constexpr int kTernThreads = 256;
constexpr int kChunk = kTernThreads * 16;   // weights per block iteration
constexpr int kMaxBlocks = 4096;

struct TernWorkspace {
    double p1[kMaxBlocks];     // pass-1 partial sums of |W|
    double p2[kMaxBlocks];     // pass-2 partial masked sums
    uint64_t cnt[kMaxBlocks];  // pass-2 partial counts
};

// Pass 1 of block `bid` out of `nblk` cooperating blocks: float64 partial sum of |W| -> partial[bid].
__device__ __forceinline__ void abs_sum_body(const float* __restrict__ W, int64_t n, double* __restrict__ partial,
                                             int bid, int nblk) {
    __shared__ double scratch[16];
    const int tid = threadIdx.x;
    const int64_t nfull = n / kChunk;          // chunks that need no bounds test
    double acc = 0.0;
    auto load4 = [&](int64_t c, float4* v) {
        const float4* src = reinterpret_cast<const float4*>(W + c * kChunk);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = src[j * kTernThreads + tid];
    };
    // software pipeline: the next chunk's loads are in flight while this one is summed
    int64_t c = bid;
    float4 cur[4];
    if (c < nfull) load4(c, cur);
    while (c < nfull) {
        const int64_t nx = c + nblk;
        float4 nxt[4];
        if (nx < nfull) load4(nx, nxt);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc += static_cast<double>(fabsf(cur[j].x));
            acc += static_cast<double>(fabsf(cur[j].y));
            acc += static_cast<double>(fabsf(cur[j].z));
            acc += static_cast<double>(fabsf(cur[j].w));
        }
        if (nx < nfull) {
#pragma unroll
            for (int j = 0; j < 4; ++j) cur[j] = nxt[j];
        }
        c = nx;
    }
    // ragged tail (at most one chunk), taken by one block after its full chunks
    if (nfull * kChunk < n && static_cast<int64_t>(bid) == nfull % nblk) {
        const int64_t base = nfull * kChunk;
        for (int j = 0; j < 4; ++j)
            for (int e = 0; e < 4; ++e) {
                const int64_t idx = base + static_cast<int64_t>(j * kTernThreads + tid) * 4 + e;
                if (idx < n) acc += static_cast<double>(fabsf(W[idx]));
            }
    }
    const double total = block_sum(acc, scratch);
    if (tid == 0) partial[bid] = total;
}

__global__ __launch_bounds__(kTernThreads) void abs_sum_kernel(const float* __restrict__ W, int64_t n,
                                                               double* __restrict__ partial) {
    abs_sum_body(W, n, partial, blockIdx.x, gridDim.x);
}

// Delta = (float)((double)f * S1 / n), S1 = fixed-order sum of the pass-1 partials.
__device__ __forceinline__ float delta_from_partials(const double* __restrict__ p1, int nb1, float f,
                                                     int64_t n, double* scratch) {
    double acc = 0.0;
    for (int i = threadIdx.x; i < nb1; i += blockDim.x) acc += p1[i];
    const double s1 = block_sum(acc, scratch);
    return static_cast<float>((static_cast<double>(f) * s1) / static_cast<double>(n));
}

// Fixed-order sum of the pass-2 partials of `nb2` blocks -> Delta, alpha, nnz (one block).
__device__ __forceinline__ void finalize_body(const TernWorkspace* __restrict__ ws, int nb1, int nb2,
                                              float f, int64_t n, float* __restrict__ delta,
                                              float* __restrict__ alpha, uint64_t* __restrict__ nnz) {
    __shared__ double scratch[16];
    __shared__ unsigned long long scratch_u[16];
    // all loads of the three partial arrays are issued before any sum is formed
    double a1 = 0.0, acc = 0.0;
    unsigned long long c = 0;
#pragma unroll 4
    for (int i = threadIdx.x; i < nb1; i += blockDim.x) a1 += ws->p1[i];
#pragma unroll 4
    for (int i = threadIdx.x; i < nb2; i += blockDim.x) {
        acc += ws->p2[i];
        c += ws->cnt[i];
    }
    const double s1 = block_sum(a1, scratch);
    const float d = static_cast<float>((static_cast<double>(f) * s1) / static_cast<double>(n));
    const double s = block_sum(acc, scratch);
    const unsigned long long total = block_sum(c, scratch_u);
    if (threadIdx.x == 0) {
        delta[0] = d;
        nnz[0] = total;
        alpha[0] = total ? static_cast<float>(s / static_cast<double>(total)) : 0.0f;
    }
}

__global__ __launch_bounds__(kTernThreads) void finalize_kernel(const TernWorkspace* __restrict__ ws, int nb1, int nb2,
                                                                float f, int64_t n, float* __restrict__ delta,
                                                                float* __restrict__ alpha, uint64_t* __restrict__ nnz) {
    finalize_body(ws, nb1, nb2, f, n, delta, alpha, nnz);
}

__device__ __forceinline__ uint32_t quad_or(uint32_t v) {
    // OR across the 4 lanes of a quad (DPP quad_perm [1,0,3,2] then [2,3,0,1]).
    v |= static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0xB1, 0xF, 0xF, false));
    v |= static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x4E, 0xF, 0xF, false));
    return v;
}

// Pass 2 for flat layouts: the packed word index is (flat weight index)/16.
// A wave covers 1024 consecutive weights per step with four fully coalesced
// float4 loads; the four lanes of a quad hold the 16 weights of one output
// word, which is assembled with two DPP ORs and written by the lane whose
// position in the quad equals the load index, so each wave stores 256
// contiguous bytes.
__device__ __forceinline__ void mask_pack_flat_body(
    const float* __restrict__ W, int64_t n, TernWorkspace* __restrict__ ws, int nb1, float f,
    uint32_t* __restrict__ packed, int reverse, int bid, int nblk) {
    const double* __restrict__ p1 = ws->p1;
    __shared__ double scratch[16];
    __shared__ unsigned long long scratch_u[16];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int ql = lane & 3;
    const float delta = delta_from_partials(p1, nb1, f, n, scratch);

    const int64_t nchunks = (n + kChunk - 1) / kChunk;
    const int64_t nfull = n / kChunk;   // chunks that need no bounds test
    const int64_t n4 = n >> 2;          // n % 16 == 0 here
    const int64_t nwords = n >> 4;
    double acc = 0.0;
    uint32_t count = 0;

    auto wave_base = [&](int64_t it) -> int64_t {
        const int64_t c = reverse ? (nchunks - 1 - it) : it;
        return c * kChunk + wave * 1024;   // first weight of this wave's span
    };
    auto load4 = [&](int64_t wbase, float4* v, bool guard) {
        const float4* src = reinterpret_cast<const float4*>(W + wbase);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (guard) {
                const int64_t i4 = (wbase >> 2) + j * 64 + lane;
                v[j] = (i4 < n4) ? src[j * 64 + lane] : make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                v[j] = src[j * 64 + lane];
            }
        }
    };
    auto process = [&](const float4* v, int64_t wbase, bool guard) {
        uint32_t mine = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t f0 = code_field(v[j].x, delta), f1 = code_field(v[j].y, delta);
            const uint32_t f2 = code_field(v[j].z, delta), f3 = code_field(v[j].w, delta);
            // adding +0.0 for the masked-out weights leaves the float64 sum unchanged
            acc += static_cast<double>(f0 ? fabsf(v[j].x) : 0.0f);
            acc += static_cast<double>(f1 ? fabsf(v[j].y) : 0.0f);
            acc += static_cast<double>(f2 ? fabsf(v[j].z) : 0.0f);
            acc += static_cast<double>(f3 ? fabsf(v[j].w) : 0.0f);
            count += (f0 & 1u) + (f1 & 1u) + (f2 & 1u) + (f3 & 1u);
            uint32_t word = ((f0 | (f2 << 2)) << (4 * ql)) | ((f1 | (f3 << 2)) << (16 + 4 * ql));
            word = quad_or(word);
            if (ql == j) mine = word;
        }
        const int64_t widx = (wbase >> 4) + (lane >> 2) + 16 * ql;
        if (!guard || widx < nwords) packed[widx] = mine;
    };

    // iteration `it` maps to chunk it (or nchunks-1-it when walking backwards); a chunk is ragged only
    // if it is the last one in memory order, i.e. it == nchunks-1 forwards or it == 0 backwards
    const bool has_tail = nfull < nchunks;
    const int64_t tail_it = reverse ? 0 : nchunks - 1;
    int64_t it = bid;
    if (has_tail && it == tail_it) {            // only possible for the first iteration of one block
        float4 v[4];
        const int64_t wb = wave_base(it);
        load4(wb, v, true);
        process(v, wb, true);
        it += nblk;
    }
    const int64_t it_end = (has_tail && !reverse) ? nchunks - 1 : nchunks;
    // software pipeline over the full chunks: next loads in flight while this chunk is processed
    float4 cur[4];
    if (it < it_end) load4(wave_base(it), cur, false);
    while (it < it_end) {
        const int64_t nx = it + nblk;
        float4 nxt[4];
        if (nx < it_end) load4(wave_base(nx), nxt, false);
        process(cur, wave_base(it), false);
        if (nx < it_end) {
#pragma unroll
            for (int j = 0; j < 4; ++j) cur[j] = nxt[j];
        }
        it = nx;
    }
    if (has_tail && !reverse && static_cast<int64_t>(bid) == tail_it % nblk && tail_it >= nblk) {
        float4 v[4];
        const int64_t wb = wave_base(tail_it);
        load4(wb, v, true);
        process(v, wb, true);
    }
    const double total = block_sum(acc, scratch);
    const unsigned long long ctotal = block_sum(static_cast<unsigned long long>(count), scratch_u);
    if (threadIdx.x == 0) {
        ws->p2[bid] = total;
        ws->cnt[bid] = ctotal;
    }
}

__global__ __launch_bounds__(kTernThreads) void mask_pack_flat_kernel(
    const float* __restrict__ W, int64_t n, TernWorkspace* __restrict__ ws, int nb1, float f,
    uint32_t* __restrict__ packed, int reverse) {
    mask_pack_flat_body(W, n, ws, nb1, f, packed, reverse, blockIdx.x, gridDim.x);
}

// Pass 2 for any layout: grid-stride over the output words of the normal copy (which also carry the
// masked sum and count: every weight belongs to exactly one normal word) and of the transposed copy.
//   normal:     row = filter o,        k   = (r*S+s)*C + c
//   transposed: row = input channel c, k_T = (r*S+s)*rows + o   (threads ordered with c fastest)
__device__ __forceinline__ void mask_pack_gather_body(
    const float* __restrict__ W, int rows, int C, int RS, TernWorkspace* __restrict__ ws, int nb1, float f,
    uint32_t* __restrict__ packed, int wpr, uint32_t* __restrict__ packed_T, int wprT, int bid, int nblk,
    bool only_transposed = false, int slot0 = 0) {
    __shared__ double scratch[16];
    __shared__ unsigned long long scratch_u[16];
    const int64_t n = static_cast<int64_t>(rows) * C * RS;
    const float delta = delta_from_partials(ws->p1, nb1, f, n, scratch);
    const int64_t words_n = only_transposed ? 0 : static_cast<int64_t>(rows) * wpr;
    const int64_t words_t = packed_T ? static_cast<int64_t>(C) * wprT : 0;
    const int64_t K = static_cast<int64_t>(RS) * C, KT = static_cast<int64_t>(RS) * rows;
    double acc = 0.0;
    uint32_t count = 0;
    for (int64_t id = static_cast<int64_t>(bid) * blockDim.x + threadIdx.x; id < words_n + words_t;
         id += static_cast<int64_t>(nblk) * blockDim.x) {
        uint32_t word = 0;
        if (id < words_n) {
            const int o = static_cast<int>(id / wpr), j = static_cast<int>(id % wpr);
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                const int64_t k = static_cast<int64_t>(j) * 16 + t;
                if (k < K) {
                    const int rs = static_cast<int>(k / C);
                    const int c = static_cast<int>(k - static_cast<int64_t>(rs) * C);
                    const float w = W[(static_cast<int64_t>(o) * C + c) * RS + rs];
                    const uint32_t fld = code_field(w, delta);
                    if (fld) {
                        acc += static_cast<double>(fabsf(w));
                        ++count;
                    }
                    word |= fld << ((t & 1) * 16 + (t >> 1) * 2);
                }
            }
            packed[id] = word;
        } else {
            const int64_t it = id - words_n;
            const int c = static_cast<int>(it % C), j = static_cast<int>(it / C);
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                const int64_t k = static_cast<int64_t>(j) * 16 + t;
                if (k < KT) {
                    const int rs = static_cast<int>(k / rows);
                    const int o = static_cast<int>(k - static_cast<int64_t>(rs) * rows);
                    word |= code_field(W[(static_cast<int64_t>(o) * C + c) * RS + rs], delta)
                            << ((t & 1) * 16 + (t >> 1) * 2);
                }
            }
            packed_T[static_cast<int64_t>(c) * wprT + j] = word;
        }
    }
    const double total = block_sum(acc, scratch);
    const unsigned long long ctotal = block_sum(static_cast<unsigned long long>(count), scratch_u);
    if (threadIdx.x == 0) {
        ws->p2[slot0 + bid] = total;
        ws->cnt[slot0 + bid] = ctotal;
    }
}

__global__ __launch_bounds__(kTernThreads) void mask_pack_gather_kernel(
    const float* __restrict__ W, int rows, int C, int RS, TernWorkspace* __restrict__ ws, int nb1, float f,
    uint32_t* __restrict__ packed, int wpr, uint32_t* __restrict__ packed_T, int wprT) {
    mask_pack_gather_body(W, rows, C, RS, ws, nb1, f, packed, wpr, packed_T, wprT, blockIdx.x, gridDim.x);
}

// Pass 2 for tensors with rows % 16 == 0 and C % 16 == 0 (filter banks, and matrices that also need the
// transposed copy), staged through LDS: block `bid` owns 16 consecutive filters x CT consecutive channels
// x all taps.  Its weights are 16 contiguous runs
// of CT*R*S floats, read once with coalesced float4 loads; the 2-bit fields go to LDS as bytes in memory
// order, and the words of both copies are assembled from LDS (16 byte reads per word), so no thread
// gathers from global memory.  Words written: per filter and tap CT/16 normal words; per channel and tap
// one transposed word (its 16 codes are the block's 16 filters).  Row padding words are written by the
// blocks with channel tile 0 (normal) and filter tile 0 (transposed).
constexpr int kTileRows = 16;
constexpr int kTileLdsBytes = 16 * 64 * 25;   // CT <= 64 with R*S <= 25 taps; CT <= 1024 for matrices
__host__ __device__ inline int tile_ct(int C, int RS) {
    if (RS == 1) {
        // matrices: the largest power of two up to 1024 that divides C (runs of up to 4 KB per filter)
        int ct = 16;
        while (ct < 1024 && C % (2 * ct) == 0) ct *= 2;
        return ct;
    }
    return (C % 64 == 0) ? 64 : (C % 32 == 0) ? 32 : 16;
}
__host__ __device__ inline bool tile_ok(int rows, int C, int RS) {
    return RS >= 1 && RS <= 25 && rows % 16 == 0 && C % 16 == 0 &&
           static_cast<int64_t>(rows / 16) * (C / tile_ct(C, RS)) <= kMaxBlocks;
}

__device__ __forceinline__ void mask_pack_tile_body(
    const float* __restrict__ W, int rows, int C, int RS, TernWorkspace* __restrict__ ws, int nb1, float f,
    uint32_t* __restrict__ packed, int wpr, uint32_t* __restrict__ packed_T, int wprT, int bid) {
    __shared__ double scratch[16];
    __shared__ unsigned long long scratch_u[16];
    __shared__ __attribute__((aligned(16))) unsigned char codes[kTileLdsBytes];
    const int64_t n = static_cast<int64_t>(rows) * C * RS;
    const float delta = delta_from_partials(ws->p1, nb1, f, n, scratch);
    const int CT = tile_ct(C, RS), ctiles = C / CT;
    const int o0 = (bid / ctiles) * kTileRows, c0 = (bid % ctiles) * CT;
    const int seg = CT * RS;                       // floats (and code bytes) per filter in this block
    const int tid = threadIdx.x;
    double acc = 0.0;
    uint32_t count = 0;
    for (int ol = 0; ol < kTileRows; ++ol) {
        const float4* src = reinterpret_cast<const float4*>(W + (static_cast<int64_t>(o0 + ol) * C + c0) * RS);
        for (int p = tid; p < seg / 4; p += kTernThreads) {
            const float4 v = src[p];
            const float w4[4] = {v.x, v.y, v.z, v.w};
            uint32_t four = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t fld = code_field(w4[e], delta);
                if (fld) {
                    acc += static_cast<double>(fabsf(w4[e]));
                    ++count;
                }
                four |= fld << (8 * e);
            }
            *reinterpret_cast<uint32_t*>(codes + ol * seg + 4 * p) = four;
        }
    }
    __syncthreads();
    // normal copy: word (ol, rs, g) holds channels c0 + 16g .. +15 of tap rs
    const int groups = CT / 16;
    for (int wi = tid; wi < kTileRows * RS * groups; wi += kTernThreads) {
        const int g = wi % groups, t1 = wi / groups;
        const int rs = t1 % RS, ol = t1 / RS;
        const unsigned char* src = codes + ol * seg + (16 * g) * RS + rs;
        uint32_t word = 0;
#pragma unroll
        for (int t = 0; t < 16; ++t) word |= static_cast<uint32_t>(src[t * RS]) << ((t & 1) * 16 + (t >> 1) * 2);
        packed[static_cast<int64_t>(o0 + ol) * wpr + (rs * C + c0) / 16 + g] = word;
    }
    if (c0 == 0) {
        const int kw = RS * C / 16, pad = wpr - kw;
        for (int wi = tid; wi < kTileRows * pad; wi += kTernThreads)
            packed[static_cast<int64_t>(o0 + wi / pad) * wpr + kw + wi % pad] = 0u;
    }
    if (packed_T) {
        // transposed copy: word (cl, rs) holds filters o0 .. o0+15
        for (int wi = tid; wi < CT * RS; wi += kTernThreads) {
            const int rs = wi % RS, cl = wi / RS;
            const unsigned char* src = codes + cl * RS + rs;
            uint32_t word = 0;
#pragma unroll
            for (int t = 0; t < 16; ++t) word |= static_cast<uint32_t>(src[t * seg]) << ((t & 1) * 16 + (t >> 1) * 2);
            packed_T[static_cast<int64_t>(c0 + cl) * wprT + (rs * rows + o0) / 16] = word;
        }
        if (o0 == 0) {
            const int kw = RS * rows / 16, pad = wprT - kw;
            for (int wi = tid; wi < CT * pad; wi += kTernThreads)
                packed_T[static_cast<int64_t>(c0 + wi / pad) * wprT + kw + wi % pad] = 0u;
        }
    }
    const double total = block_sum(acc, scratch);
    const unsigned long long ctotal = block_sum(static_cast<unsigned long long>(count), scratch_u);
    if (tid == 0) {
        ws->p2[bid] = total;
        ws->cnt[bid] = ctotal;
    }
}

__global__ __launch_bounds__(kTernThreads) void mask_pack_tile_kernel(
    const float* __restrict__ W, int rows, int C, int RS, TernWorkspace* __restrict__ ws, int nb1, float f,
    uint32_t* __restrict__ packed, int wpr, uint32_t* __restrict__ packed_T, int wprT) {
    mask_pack_tile_body(W, rows, C, RS, ws, nb1, f, packed, wpr, packed_T, wprT, blockIdx.x);
}

// ---- several tensors per launch --------------------------------------------------------------
// The weight tensors of a network are small (at most a few MB): ternarizing them one call at a time is
// bound by launch latency and by kernels too small to fill the chip.  The batch entry point runs the same
// three passes once for up to kBatchMax tensors; a block finds its tensor in a table passed by value.
constexpr int kBatchMax = 32;
struct BatchItem {
    const float* W;
    uint32_t* packed;
    uint32_t* packed_T;
    float* delta;
    float* alpha;
    uint64_t* nnz;
    int32_t rows, C, RS, wpr, wprT;
    int32_t nb1, nb2;           // blocks of pass 1 / pass 2 working on this tensor
    int32_t tiled;              // pass 2 through the LDS-staged tile body
    int32_t flat_blocks;        // > 0: flat layout, the first flat_blocks pass-2 blocks stream W, the rest gather the transposed copy
    int32_t first1, first2;     // index of its first block in the pass-1 / pass-2 launch
    // several groups (one Delta, alpha per `rows / groups` filters): the tensor takes no part in the three per-layer
    // launches (nb1 = nb2 = 0) but in the two per-group ones
    int32_t groups;
    int32_t firstg, firstp;     // index of its first block in the group-statistics / the code-packing launch
    int32_t npb;                // its blocks in the code-packing launch
};
struct BatchTable {
    BatchItem item[kBatchMax];
    int32_t count;
    float f;
};

__device__ __forceinline__ int batch_find(const BatchTable& tb, int block, bool pass2) {
    int i = 0;
    while (i + 1 < tb.count && block >= (pass2 ? tb.item[i + 1].first2 : tb.item[i + 1].first1)) ++i;
    return i;
}
// the same for the two per-group launches (a tensor without blocks in a launch shares its first index with its
// successor and is passed over)
__device__ __forceinline__ int batch_find_group(const BatchTable& tb, int block, bool pack) {
    int i = 0;
    while (i + 1 < tb.count && block >= (pack ? tb.item[i + 1].firstp : tb.item[i + 1].firstg)) ++i;
    return i;
}

__global__ __launch_bounds__(kTernThreads) void batch_abs_sum_kernel(const BatchTable tb, TernWorkspace* __restrict__ ws) {
    const int i = batch_find(tb, blockIdx.x, false);
    const BatchItem& it = tb.item[i];
    abs_sum_body(it.W, static_cast<int64_t>(it.rows) * it.C * it.RS, ws[i].p1, blockIdx.x - it.first1, it.nb1);
}

__global__ __launch_bounds__(kTernThreads) void batch_mask_pack_kernel(const BatchTable tb, TernWorkspace* __restrict__ ws) {
    const int i = batch_find(tb, blockIdx.x, true);
    const BatchItem& it = tb.item[i];
    if (it.flat_blocks > 0) {
        const int local = blockIdx.x - it.first2;
        const int64_t n = static_cast<int64_t>(it.rows) * it.C;
        if (local < it.flat_blocks)
            mask_pack_flat_body(it.W, n, ws + i, it.nb1, tb.f, it.packed, 1, local, it.flat_blocks);
        else
            mask_pack_gather_body(it.W, it.rows, it.C, it.RS, ws + i, it.nb1, tb.f, it.packed, it.wpr, it.packed_T, it.wprT,
                                  local - it.flat_blocks, it.nb2 - it.flat_blocks, true, it.flat_blocks);
    } else if (it.tiled)
        mask_pack_tile_body(it.W, it.rows, it.C, it.RS, ws + i, it.nb1, tb.f, it.packed, it.wpr, it.packed_T, it.wprT,
                            blockIdx.x - it.first2);
    else
        mask_pack_gather_body(it.W, it.rows, it.C, it.RS, ws + i, it.nb1, tb.f, it.packed, it.wpr, it.packed_T, it.wprT,
                              blockIdx.x - it.first2, it.nb2);
}

__global__ __launch_bounds__(kTernThreads) void batch_finalize_kernel(const BatchTable tb, const TernWorkspace* __restrict__ ws) {
    const BatchItem& it = tb.item[blockIdx.x];
    if (it.groups > 1) return;      // per-group tensors were finished by batch_group_stats_kernel
    finalize_body(ws + blockIdx.x, it.nb1, it.nb2, tb.f, static_cast<int64_t>(it.rows) * it.C * it.RS, it.delta, it.alpha,
                  it.nnz);
}

// One block per group: both passes over the group's contiguous weights.
__device__ __forceinline__ void group_stats_body(const float* __restrict__ W, int64_t n_per_group, float f,
                                                 float* __restrict__ delta, float* __restrict__ alpha,
                                                 uint64_t* __restrict__ nnz, int group) {
    __shared__ double scratch[16];
    __shared__ unsigned long long scratch_u[16];
    const float* seg = W + static_cast<int64_t>(group) * n_per_group;
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < n_per_group; i += blockDim.x) acc += static_cast<double>(fabsf(seg[i]));
    const double s1 = block_sum(acc, scratch);
    const float d = static_cast<float>((static_cast<double>(f) * s1) / static_cast<double>(n_per_group));
    acc = 0.0;
    uint32_t count = 0;
    for (int64_t i = threadIdx.x; i < n_per_group; i += blockDim.x) {
        const float a = fabsf(seg[i]);
        if (a > d) {
            acc += static_cast<double>(a);
            ++count;
        }
    }
    const double s = block_sum(acc, scratch);
    const unsigned long long total = block_sum(static_cast<unsigned long long>(count), scratch_u);
    if (threadIdx.x == 0) {
        delta[group] = d;
        nnz[group] = total;
        alpha[group] = total ? static_cast<float>(s / static_cast<double>(total)) : 0.0f;
    }
}

__global__ __launch_bounds__(kTernThreads) void group_stats_kernel(
    const float* __restrict__ W, int64_t n_per_group, float f,
    float* __restrict__ delta, float* __restrict__ alpha, uint64_t* __restrict__ nnz) {
    group_stats_body(W, n_per_group, f, delta, alpha, nnz, blockIdx.x);
}

__global__ __launch_bounds__(kTernThreads) void batch_group_stats_kernel(const BatchTable tb) {
    const int i = batch_find_group(tb, blockIdx.x, false);
    const BatchItem& it = tb.item[i];
    group_stats_body(it.W, static_cast<int64_t>(it.rows) * it.C * it.RS / it.groups, tb.f, it.delta, it.alpha, it.nnz,
                     blockIdx.x - it.firstg);
}

// ---- sign binarization of the binary-weight comparison (Sec. 3) ------------------------------------------
// alpha of one group per block (float64 sum in a fixed order); used for several groups, where a group is small.
__global__ __launch_bounds__(kTernThreads) void group_abs_mean_kernel(const float* __restrict__ W, int64_t n_per_group,
                                                                      float* __restrict__ alpha) {
    __shared__ double scratch[16];
    const float* seg = W + static_cast<int64_t>(blockIdx.x) * n_per_group;
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < n_per_group; i += blockDim.x) acc += static_cast<double>(fabsf(seg[i]));
    const double s1 = block_sum(acc, scratch);
    if (threadIdx.x == 0) alpha[blockIdx.x] = static_cast<float>(s1 / static_cast<double>(n_per_group));
}

// alpha of a whole tensor from the pass-1 partial sums of abs_sum_kernel (one block).
__global__ __launch_bounds__(kTernThreads) void abs_mean_finalize_kernel(const double* __restrict__ p1, int nb1, int64_t n,
                                                                         float* __restrict__ alpha) {
    __shared__ double scratch[16];
    double acc = 0.0;
    for (int i = threadIdx.x; i < nb1; i += blockDim.x) acc += p1[i];
    const double s1 = block_sum(acc, scratch);
    if (threadIdx.x == 0) alpha[0] = static_cast<float>(s1 / static_cast<double>(n));
}

// 1-bit sign codes of a matrix whose rows need no padding (K % 128 == 0): a wave takes 64 consecutive weights
// per step, lane l reading the weight whose code lands in bit l of the two output words (even k first, then
// odd k, per word), so that the wave's ballot is the pair of words.
__global__ __launch_bounds__(256) void sign_pack_flat_kernel(const float* __restrict__ W, int64_t npairs,
                                                             uint64_t* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = (static_cast<int64_t>(gridDim.x) * blockDim.x) >> 6;
    const int l = lane & 31;
    const int koff = (lane >> 5) * 32 + (l < 16 ? 2 * l : 2 * (l - 16) + 1);
    for (int64_t p = wave; p < npairs; p += nwaves) {
        const unsigned long long m = __ballot(W[p * 64 + koff] < 0.0f);
        if (lane == 0) out[p] = m;
    }
}

// 1-bit sign codes, one thread per output word (32 weights): k = (r*S+s)*C + c of filter `row`.
__global__ __launch_bounds__(256) void sign_pack_kernel(const float* __restrict__ W, int rows, int C, int RS,
                                                        uint32_t* __restrict__ out, int wpr) {
    const int64_t id = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (id >= static_cast<int64_t>(rows) * wpr) return;
    const int row = static_cast<int>(id / wpr), j = static_cast<int>(id % wpr);
    const int64_t K = static_cast<int64_t>(RS) * C;
    uint32_t word = 0;
#pragma unroll 8
    for (int t = 0; t < 32; ++t) {
        const int64_t k = static_cast<int64_t>(j) * 32 + t;
        if (k < K) {
            const int rs = static_cast<int>(k / C);
            const int c = static_cast<int>(k - static_cast<int64_t>(rs) * C);
            const float w = W[(static_cast<int64_t>(row) * C + c) * RS + rs];
            word |= (w < 0.0f ? 1u : 0u) << ((t & 1) * 16 + (t >> 1));
        }
    }
    out[id] = word;
}

// Codes for any layout.  One thread per output word.
//   normal:     out row = filter o,        k   = (r*S+s)*C + c
//   transposed: out row = input channel c, k_T = (r*S+s)*rows + o
// Threads are ordered so that neighbouring threads read neighbouring source
// weights where the layout allows it.
__device__ __forceinline__ void pack_gather_body(
    const float* __restrict__ W, int rows, int C, int RS, const float* __restrict__ delta,
    int rows_per_group, uint32_t* __restrict__ out, int wpr, int transposed, int64_t id) {
    int64_t out_rows = transposed ? C : rows;
    if (id >= out_rows * wpr) return;
    int row, j;
    if (transposed) {
        row = static_cast<int>(id % C);   // input channel, fastest across threads
        j = static_cast<int>(id / C);
    } else {
        row = static_cast<int>(id / wpr);
        j = static_cast<int>(id % wpr);
    }
    const int64_t K = transposed ? static_cast<int64_t>(RS) * rows : static_cast<int64_t>(RS) * C;
    uint32_t word = 0;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int64_t k = static_cast<int64_t>(j) * 16 + t;
        if (k < K) {
            int o, c, rs;
            if (transposed) {
                rs = static_cast<int>(k / rows);
                o = static_cast<int>(k - static_cast<int64_t>(rs) * rows);
                c = row;
            } else {
                rs = static_cast<int>(k / C);
                c = static_cast<int>(k - static_cast<int64_t>(rs) * C);
                o = row;
            }
            const float w = W[(static_cast<int64_t>(o) * C + c) * RS + rs];
            const uint32_t fld = code_field(w, delta[o / rows_per_group]);
            word |= fld << ((t & 1) * 16 + (t >> 1) * 2);
        }
    }
    out[static_cast<int64_t>(row) * wpr + j] = word;
}

__global__ __launch_bounds__(256) void pack_gather_kernel(
    const float* __restrict__ W, int rows, int C, int RS, const float* __restrict__ delta,
    int rows_per_group, uint32_t* __restrict__ out, int wpr, int transposed) {
    pack_gather_body(W, rows, C, RS, delta, rows_per_group, out, wpr, transposed,
                     static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x);
}

// Per-group tensors of a multi-tensor call: the words of the normal copy, then those of the transposed copy.
__global__ __launch_bounds__(256) void batch_pack_gather_kernel(const BatchTable tb) {
    const int i = batch_find_group(tb, blockIdx.x, true);
    const BatchItem& it = tb.item[i];
    const int64_t id = static_cast<int64_t>(blockIdx.x - it.firstp) * blockDim.x + threadIdx.x;
    const int64_t words_n = static_cast<int64_t>(it.rows) * it.wpr;
    const int rpg = it.rows / it.groups;
    if (id < words_n)
        pack_gather_body(it.W, it.rows, it.C, it.RS, it.delta, rpg, it.packed, it.wpr, 0, id);
    else if (it.packed_T)
        pack_gather_body(it.W, it.rows, it.C, it.RS, it.delta, rpg, it.packed_T, it.wprT, 1, id - words_n);
}

__global__ __launch_bounds__(256) void unpack_i8_kernel(const uint32_t* __restrict__ packed, int rows,
                                                        int64_t K, int wpr, int8_t* __restrict__ codes) {
    const int64_t id = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (id >= static_cast<int64_t>(rows) * K) return;
    const int64_t row = id / K, k = id % K;
    const uint32_t word = packed[row * wpr + (k >> 4)];
    const int t = static_cast<int>(k & 15);
    const uint32_t fld = (word >> ((t & 1) * 16 + (t >> 1) * 2)) & 3u;
    codes[id] = (fld & 1u) ? ((fld & 2u) ? -1 : 1) : 0;
}

}  // namespace twn

using namespace twn;

extern "C" size_t twn_ternarize_workspace_bytes(const twn_weight_desc* wd, int32_t groups) {
    if (!wd || groups < 1) return 0;
    return sizeof(TernWorkspace);
}

// Host-side argument checks shared by twn_ternarize and twn_ternarize_static (no GPU call).
static int32_t ternarize_check(const float* W, const twn_weight_desc* wd, int32_t groups, float delta_factor,
                               const uint32_t* packed, const uint32_t* packed_T, const float* delta,
                               const float* alpha, const uint64_t* nnz) {
    if (!W || !wd || !packed || !delta || !alpha || !nnz) return TWN_ERR_NULL;
    if (wd->rows <= 0 || wd->C <= 0 || wd->R <= 0 || wd->S <= 0) return TWN_ERR_SHAPE;
    if (groups < 1 || wd->rows % groups != 0) return TWN_ERR_SHAPE;
    if (!(delta_factor > 0.0f) || delta_factor > 1.0f) return TWN_ERR_SHAPE;
    const int64_t RS = static_cast<int64_t>(wd->R) * wd->S;
    const int64_t K = RS * wd->C;
    const int64_t KT = RS * wd->rows;
    const int64_t n = K * wd->rows;
    if (RS > (1 << 15) || K >= (1LL << 31) || KT >= (1LL << 31) || n >= (1LL << 40)) return TWN_ERR_SHAPE;
    if (!aligned(W, 16) || !aligned(packed, 16) || (packed_T && !aligned(packed_T, 16))) return TWN_ERR_ALIGN;
    return TWN_OK;
}

// Blocks of pass 1 for a tensor of n weights (two persistent blocks per CU measured best with the prefetch);
// the parameter update that leaves pass-1 sums behind uses the same partition.
static int pass1_blocks(int64_t n) {
    const int64_t nchunks = (n + kChunk - 1) / kChunk;
    int want = env_int("TWN_TERN_BLOCKS", 512);
    if (want < 1) want = 1;
    if (want > kMaxBlocks) want = kMaxBlocks;
    return static_cast<int>(nchunks < want ? nchunks : want);
}

// Launches of one ternarization; `workspace` is device memory of at least sizeof(TernWorkspace) bytes, either
// the caller's (twn_ternarize) or the library's own per-device array (twn_ternarize_static).
static int32_t ternarize_impl(const float* W, const twn_weight_desc* wd, int32_t groups,
                              float delta_factor, uint32_t* packed, uint32_t* packed_T,
                              float* delta, float* alpha, uint64_t* nnz,
                              void* workspace, size_t workspace_bytes, void* stream, bool presummed = false) {
    const int32_t rc = ternarize_check(W, wd, groups, delta_factor, packed, packed_T, delta, alpha, nnz);
    if (rc != TWN_OK) return rc;
    if (presummed && groups != 1) return TWN_ERR_UNSUPPORTED;
    const int64_t RS = static_cast<int64_t>(wd->R) * wd->S;
    const int64_t K = RS * wd->C;
    const int64_t KT = RS * wd->rows;
    const int64_t n = K * wd->rows;
    if (!workspace || workspace_bytes < sizeof(TernWorkspace) || !aligned(workspace, 8)) return TWN_ERR_WORKSPACE;

    hipStream_t st = as_stream(stream);
    const int wpr = static_cast<int>(twn_packed_words_per_row(K));
    const int wprT = static_cast<int>(twn_packed_words_per_row(KT));
    const int rows_per_group = wd->rows / groups;

    if (groups == 1) {
        TernWorkspace* ws = static_cast<TernWorkspace*>(workspace);
        const int nb = pass1_blocks(n);
        if (!presummed) abs_sum_kernel<<<nb, kTernThreads, 0, st>>>(W, n, ws->p1);
        // matrices stream through the flat kernel; when the transposed copy is wanted too, the tile kernel
        // writes both from one read of W instead of a second, gathering pass
        const bool flat = (RS == 1) && (K % 128 == 0) && !(packed_T && tile_ok(wd->rows, wd->C, 1));
        if (flat) {
            const int reverse = env_int("TWN_TERN_REVERSE", 1);
            mask_pack_flat_kernel<<<nb, kTernThreads, 0, st>>>(W, n, ws, nb, delta_factor, packed, reverse);
            finalize_kernel<<<1, kTernThreads, 0, st>>>(ws, nb, nb, delta_factor, n, delta, alpha, nnz);
            if (packed_T) {
                const int64_t words = static_cast<int64_t>(wd->C) * wprT;
                pack_gather_kernel<<<static_cast<unsigned>((words + 255) / 256), 256, 0, st>>>(
                    W, wd->rows, wd->C, static_cast<int>(RS), delta, rows_per_group, packed_T, wprT, 1);
            }
        } else {
            const int64_t words = static_cast<int64_t>(wd->rows) * wpr +
                                  (packed_T ? static_cast<int64_t>(wd->C) * wprT : 0);
            int64_t nb2 = (words + kTernThreads - 1) / kTernThreads;
            if (nb2 > kMaxBlocks) nb2 = kMaxBlocks;
            if (tile_ok(wd->rows, wd->C, static_cast<int>(RS))) {
                nb2 = static_cast<int64_t>(wd->rows / kTileRows) * (wd->C / tile_ct(wd->C, static_cast<int>(RS)));
                mask_pack_tile_kernel<<<static_cast<unsigned>(nb2), kTernThreads, 0, st>>>(
                    W, wd->rows, wd->C, static_cast<int>(RS), ws, nb, delta_factor, packed, wpr, packed_T, wprT);
            } else
            mask_pack_gather_kernel<<<static_cast<unsigned>(nb2), kTernThreads, 0, st>>>(
                W, wd->rows, wd->C, static_cast<int>(RS), ws, nb, delta_factor, packed, wpr, packed_T, wprT);
            finalize_kernel<<<1, kTernThreads, 0, st>>>(ws, nb, static_cast<int>(nb2), delta_factor, n, delta, alpha,
                                                        nnz);
        }
    } else {
        group_stats_kernel<<<groups, kTernThreads, 0, st>>>(W, n / groups, delta_factor, delta, alpha, nnz);
        const int64_t words = static_cast<int64_t>(wd->rows) * wpr;
        pack_gather_kernel<<<static_cast<unsigned>((words + 255) / 256), 256, 0, st>>>(
            W, wd->rows, wd->C, static_cast<int>(RS), delta, rows_per_group, packed, wpr, 0);
        if (packed_T) {
            const int64_t wordsT = static_cast<int64_t>(wd->C) * wprT;
            pack_gather_kernel<<<static_cast<unsigned>((wordsT + 255) / 256), 256, 0, st>>>(
                W, wd->rows, wd->C, static_cast<int>(RS), delta, rows_per_group, packed_T, wprT, 1);
        }
    }
    return launch_status();
}

extern "C" int32_t twn_ternarize(const float* W, const twn_weight_desc* wd, int32_t groups,
                                 float delta_factor, uint32_t* packed, uint32_t* packed_T,
                                 float* delta, float* alpha, uint64_t* nnz,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    return ternarize_impl(W, wd, groups, delta_factor, packed, packed_T, delta, alpha, nnz, workspace, workspace_bytes,
                          stream);
}

// ---- parameter update fused with pass 1 of the next ternarization (Alg. 1 step 10; Sec. 2.4; Table 1) --------
// One read of W, V, dW and one write of W, V per weight (20 bytes); the float64 sum of |W| after the update is
// accumulated chunk by chunk and element by element exactly as abs_sum_body does it, so that the partial sums
// (and with them Delta of the ternarization that follows) are bit-identical to a separate pass over the updated
// tensor, which would cost 4 more bytes per weight.
__global__ __launch_bounds__(kTernThreads) void sgd_update_kernel(float* __restrict__ W, float* __restrict__ V,
                                                                  const float* __restrict__ dW, int64_t n, float lr,
                                                                  float momentum, float wd, double* __restrict__ partial) {
    __shared__ double scratch[16];
    const int tid = threadIdx.x;
    const int bid = blockIdx.x, nblk = gridDim.x;
    const int64_t nfull = n / kChunk;
    double acc = 0.0;
    auto load4 = [&](const float* p, int64_t c, float4* v) {
        const float4* src = reinterpret_cast<const float4*>(p + c * kChunk);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = src[j * kTernThreads + tid];
    };
    auto update = [&](float& w, float& v, float g) {
        g = fmaf(wd, w, g);
        v = fmaf(momentum, v, g);
        w = fmaf(-lr, v, w);
        acc += static_cast<double>(fabsf(w));
    };
    int64_t c = bid;
    float4 w4[4], v4[4], g4[4];
    if (c < nfull) {
        load4(W, c, w4);
        load4(V, c, v4);
        load4(dW, c, g4);
    }
    while (c < nfull) {
        const int64_t nx = c + nblk;
        float4 wn[4], vn[4], gn[4];
        if (nx < nfull) {
            load4(W, nx, wn);
            load4(V, nx, vn);
            load4(dW, nx, gn);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            update(w4[j].x, v4[j].x, g4[j].x);
            update(w4[j].y, v4[j].y, g4[j].y);
            update(w4[j].z, v4[j].z, g4[j].z);
            update(w4[j].w, v4[j].w, g4[j].w);
        }
        float4* wdst = reinterpret_cast<float4*>(W + c * kChunk);
        float4* vdst = reinterpret_cast<float4*>(V + c * kChunk);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            wdst[j * kTernThreads + tid] = w4[j];
            vdst[j * kTernThreads + tid] = v4[j];
        }
        if (nx < nfull) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                w4[j] = wn[j];
                v4[j] = vn[j];
                g4[j] = gn[j];
            }
        }
        c = nx;
    }
    // ragged tail (at most one chunk), taken by the block abs_sum_body gives it to, in its element order
    if (nfull * kChunk < n && static_cast<int64_t>(bid) == nfull % nblk) {
        const int64_t base = nfull * kChunk;
        for (int j = 0; j < 4; ++j)
            for (int e = 0; e < 4; ++e) {
                const int64_t idx = base + static_cast<int64_t>(j * kTernThreads + tid) * 4 + e;
                if (idx < n) {
                    float w = W[idx], v = V[idx];
                    update(w, v, dW[idx]);
                    W[idx] = w;
                    V[idx] = v;
                }
            }
    }
    const double total = block_sum(acc, scratch);
    if (partial && tid == 0) partial[bid] = total;
}

extern "C" int32_t twn_sgd_update(float* W, float* V, const float* dW, int64_t n, float lr, float momentum,
                                  float weight_decay, void* tern_workspace, size_t workspace_bytes, void* stream) {
    if (!W || !V || !dW) return TWN_ERR_NULL;
    if (n <= 0 || n >= (1LL << 40)) return TWN_ERR_SHAPE;
    if (!(lr == lr) || !(momentum == momentum) || !(weight_decay == weight_decay)) return TWN_ERR_SHAPE;
    if (!aligned(W, 16) || !aligned(V, 16) || !aligned(dW, 16)) return TWN_ERR_ALIGN;
    if (tern_workspace && (workspace_bytes < sizeof(TernWorkspace) || !aligned(tern_workspace, 8))) return TWN_ERR_WORKSPACE;
    TernWorkspace* ws = static_cast<TernWorkspace*>(tern_workspace);
    sgd_update_kernel<<<pass1_blocks(n), kTernThreads, 0, as_stream(stream)>>>(W, V, dW, n, lr, momentum, weight_decay,
                                                                              ws ? ws->p1 : nullptr);
    return launch_status();
}

extern "C" int32_t twn_ternarize_presummed(const float* W, const twn_weight_desc* wd, float delta_factor,
                                           uint32_t* packed, uint32_t* packed_T, float* delta, float* alpha,
                                           uint64_t* nnz, void* workspace, size_t workspace_bytes, void* stream) {
    return ternarize_impl(W, wd, 1, delta_factor, packed, packed_T, delta, alpha, nnz, workspace, workspace_bytes, stream,
                          true);
}

extern "C" size_t twn_binarize_workspace_bytes(const twn_weight_desc* wd, int32_t groups) {
    (void)groups;
    if (!wd) return 0;
    return sizeof(TernWorkspace);
}

extern "C" int32_t twn_binarize(const float* W, const twn_weight_desc* wd, int32_t groups, uint32_t* packed1,
                                float* alpha, void* workspace, size_t workspace_bytes, void* stream) {
    if (!W || !wd || !packed1 || !alpha) return TWN_ERR_NULL;
    if (wd->rows <= 0 || wd->C <= 0 || wd->R <= 0 || wd->S <= 0) return TWN_ERR_SHAPE;
    if (groups < 1 || wd->rows % groups != 0) return TWN_ERR_SHAPE;
    const int64_t RS = static_cast<int64_t>(wd->R) * wd->S;
    const int64_t K = RS * wd->C;
    const int64_t n = K * wd->rows;
    if (RS > (1 << 15) || K >= (1LL << 31) || n >= (1LL << 40)) return TWN_ERR_SHAPE;
    if (!aligned(W, 16) || !aligned(packed1, 16)) return TWN_ERR_ALIGN;
    if (!workspace || workspace_bytes < sizeof(TernWorkspace) || !aligned(workspace, 8)) return TWN_ERR_WORKSPACE;
    hipStream_t st = as_stream(stream);
    if (groups == 1) {
        TernWorkspace* ws = static_cast<TernWorkspace*>(workspace);
        const int nb = pass1_blocks(n);
        abs_sum_kernel<<<nb, kTernThreads, 0, st>>>(W, n, ws->p1);
        abs_mean_finalize_kernel<<<1, kTernThreads, 0, st>>>(ws->p1, nb, n, alpha);
    } else {
        group_abs_mean_kernel<<<groups, kTernThreads, 0, st>>>(W, n / groups, alpha);
    }
    const int wpr = static_cast<int>(twn_packed1_words_per_row(K));
    const int64_t words = static_cast<int64_t>(wd->rows) * wpr;
    if (RS == 1 && K % 128 == 0) {
        const int64_t npairs = n / 64;
        const int64_t blocks = (npairs + 3) / 4 < 4096 ? (npairs + 3) / 4 : 4096;
        sign_pack_flat_kernel<<<static_cast<unsigned>(blocks), 256, 0, st>>>(W, npairs, reinterpret_cast<uint64_t*>(packed1));
    } else {
        sign_pack_kernel<<<static_cast<unsigned>((words + 255) / 256), 256, 0, st>>>(W, wd->rows, wd->C,
                                                                                      static_cast<int>(RS), packed1, wpr);
    }
    return launch_status();
}

// ---- the entry point that allocates nothing -------------------------------------------------------------
// The per-block partial sums of twn_ternarize live in a file-scope device array instead of a caller
// workspace.  Every GPU the library runs on holds its own copy of the array at its own address: the
// address is looked up once per device (with that device current) and only that pointer is ever handed
// to kernels.  Nothing in the array has to start at zero: every partial a pass reads was written by the
// pass before it in the same call.
namespace twn {
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[sizeof(TernWorkspace)];
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kStaticMaxDevices];      // per device: address of `scratch` there, null until looked up
}  // namespace twn

extern "C" size_t twn_ternarize_static_scratch_bytes(void) { return sizeof(TernWorkspace); }

extern "C" int32_t twn_ternarize_static(const float* W, const twn_weight_desc* wd, int32_t groups,
                                        float delta_factor, uint32_t* packed, uint32_t* packed_T,
                                        float* delta, float* alpha, uint64_t* nnz, void* stream) {
    // every check that needs no GPU comes first; tensors beyond the 2^40 weights the fixed array is specified
    // for are rejected here with TWN_ERR_SHAPE
    const int32_t rc = ternarize_check(W, wd, groups, delta_factor, packed, packed_T, delta, alpha, nnz);
    if (rc != TWN_OK) return rc;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return TWN_ERR_HIP;
    if (dev < 0 || dev >= kStaticMaxDevices) return TWN_ERR_UNSUPPORTED;
    void* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TWN_ERR_HIP;
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    return ternarize_impl(W, wd, groups, delta_factor, packed, packed_T, delta, alpha, nnz, ptr, sizeof(TernWorkspace),
                          stream);
}

extern "C" size_t twn_ternarize_batch_workspace_bytes(int32_t count) {
    if (count < 1 || count > kBatchMax) return 0;
    return static_cast<size_t>(count) * sizeof(TernWorkspace);
}

extern "C" int32_t twn_ternarize_batch(const twn_ternarize_item* items, int32_t count, float delta_factor,
                                       void* workspace, size_t workspace_bytes, void* stream) {
    if (!items) return TWN_ERR_NULL;
    if (count < 1 || count > kBatchMax) return TWN_ERR_SHAPE;
    if (!(delta_factor > 0.0f) || delta_factor > 1.0f) return TWN_ERR_SHAPE;
    if (!workspace || workspace_bytes < static_cast<size_t>(count) * sizeof(TernWorkspace) || !aligned(workspace, 8))
        return TWN_ERR_WORKSPACE;
    BatchTable tb{};
    tb.count = count;
    tb.f = delta_factor;
    int64_t total_n = 0;
    for (int i = 0; i < count; ++i) {
        const twn_ternarize_item& in = items[i];
        if (!in.W || !in.packed || !in.delta || !in.alpha || !in.nnz) return TWN_ERR_NULL;
        const twn_weight_desc& wd = in.wd;
        if (wd.rows <= 0 || wd.C <= 0 || wd.R <= 0 || wd.S <= 0) return TWN_ERR_SHAPE;
        const int64_t RS = static_cast<int64_t>(wd.R) * wd.S;
        const int64_t K = RS * wd.C, KT = RS * wd.rows, n = K * wd.rows;
        if (RS > (1 << 15) || K >= (1LL << 31) || KT >= (1LL << 31) || n >= (1LL << 40)) return TWN_ERR_SHAPE;
        if (!aligned(in.W, 16) || !aligned(in.packed, 16) || (in.packed_T && !aligned(in.packed_T, 16))) return TWN_ERR_ALIGN;
        if (in.groups < 1 || wd.rows % in.groups != 0) return TWN_ERR_SHAPE;
        if (in.groups == 1) total_n += n;
    }
    if (total_n == 0) total_n = 1;      // only per-group tensors
    // blocks are shared out in proportion to the tensor sizes: about 1024 per pass in total
    int first1 = 0, first2 = 0;
    int64_t firstg = 0, firstp = 0;
    for (int i = 0; i < count; ++i) {
        const twn_ternarize_item& in = items[i];
        const twn_weight_desc& wd = in.wd;
        const int64_t RS = static_cast<int64_t>(wd.R) * wd.S;
        const int64_t K = RS * wd.C, KT = RS * wd.rows, n = K * wd.rows;
        BatchItem& it = tb.item[i];
        it.W = in.W; it.packed = in.packed; it.packed_T = in.packed_T;
        it.delta = in.delta; it.alpha = in.alpha; it.nnz = in.nnz;
        it.rows = wd.rows; it.C = wd.C; it.RS = static_cast<int32_t>(RS);
        it.wpr = static_cast<int32_t>(twn_packed_words_per_row(K));
        it.wprT = static_cast<int32_t>(twn_packed_words_per_row(KT));
        it.groups = in.groups;
        it.firstg = static_cast<int32_t>(firstg);
        it.firstp = static_cast<int32_t>(firstp);
        it.npb = 0;
        if (in.groups > 1) {
            // one block per group for the statistics, one thread per output word for the codes
            const int64_t words = static_cast<int64_t>(wd.rows) * it.wpr + (in.packed_T ? static_cast<int64_t>(wd.C) * it.wprT : 0);
            it.npb = static_cast<int32_t>((words + 255) / 256);
            firstg += in.groups;
            firstp += it.npb;
            if (firstg >= (1LL << 30) || firstp >= (1LL << 30)) return TWN_ERR_SHAPE;
            it.nb1 = it.nb2 = 0;
            it.tiled = it.flat_blocks = 0;
            it.first1 = first1;
            it.first2 = first2;
            continue;
        }
        int64_t share = (1024 * n + total_n - 1) / total_n;
        if (share < 1) share = 1;
        const int64_t nchunks = (n + kChunk - 1) / kChunk;
        it.nb1 = static_cast<int32_t>(nchunks < share ? nchunks : share);
        const int64_t words = static_cast<int64_t>(wd.rows) * it.wpr + (in.packed_T ? static_cast<int64_t>(wd.C) * it.wprT : 0);
        int64_t nb2 = (words + kTernThreads - 1) / kTernThreads;
        if (nb2 > 4 * share) nb2 = 4 * share;
        if (nb2 > kMaxBlocks) nb2 = kMaxBlocks;
        if (it.nb1 > kMaxBlocks) it.nb1 = kMaxBlocks;
        const bool flat = (RS == 1) && (K % 128 == 0) && !(in.packed_T && tile_ok(wd.rows, wd.C, 1));
        it.tiled = (!flat && tile_ok(wd.rows, wd.C, static_cast<int>(RS))) ? 1 : 0;
        if (it.tiled) nb2 = static_cast<int64_t>(wd.rows / kTileRows) * (wd.C / tile_ct(wd.C, static_cast<int>(RS)));
        it.flat_blocks = 0;
        if (flat) {
            // flat layout: the normal copy is written while W streams by; only the transposed copy gathers
            it.flat_blocks = it.nb1;
            int64_t nbT = in.packed_T ? (static_cast<int64_t>(wd.C) * it.wprT + kTernThreads - 1) / kTernThreads : 0;
            if (nbT > 4 * share) nbT = 4 * share;
            if (nbT > kMaxBlocks - it.flat_blocks) nbT = kMaxBlocks - it.flat_blocks;
            nb2 = it.flat_blocks + nbT;
        }
        it.nb2 = static_cast<int32_t>(nb2);
        it.first1 = first1;
        it.first2 = first2;
        first1 += it.nb1;
        first2 += it.nb2;
    }
    hipStream_t st = as_stream(stream);
    TernWorkspace* ws = static_cast<TernWorkspace*>(workspace);
    if (first1 > 0) {
        batch_abs_sum_kernel<<<first1, kTernThreads, 0, st>>>(tb, ws);
        batch_mask_pack_kernel<<<first2, kTernThreads, 0, st>>>(tb, ws);
        batch_finalize_kernel<<<count, kTernThreads, 0, st>>>(tb, ws);
    }
    if (firstg > 0) {
        batch_group_stats_kernel<<<static_cast<unsigned>(firstg), kTernThreads, 0, st>>>(tb);
        batch_pack_gather_kernel<<<static_cast<unsigned>(firstp), 256, 0, st>>>(tb);
    }
    return launch_status();
}

extern "C" int32_t twn_unpack_i8(const uint32_t* packed, int32_t rows, int64_t K, int8_t* codes, void* stream) {
    if (!packed || !codes) return TWN_ERR_NULL;
    if (rows <= 0 || K <= 0 || K >= (1LL << 31)) return TWN_ERR_SHAPE;
    if (!aligned(packed, 16)) return TWN_ERR_ALIGN;
    const int64_t total = static_cast<int64_t>(rows) * K;
    unpack_i8_kernel<<<static_cast<unsigned>((total + 255) / 256), 256, 0, as_stream(stream)>>>(
        packed, rows, K, static_cast<int>(twn_packed_words_per_row(K)), codes);
    return launch_status();
}
