// Internal launch interface between the C-ABI entry points and the kernels.
#pragma once

#include "twn_common.h"

namespace twn {

// One implicit-GEMM problem:  Y[m][n] = epilogue( sum_k A[m][k] * code[n][k] ).
// Rows m enumerate (batch, oh, ow) of the *output* of the gather; k enumerates
// (r, s, c) with c fastest.  A[m][k] is read from the NHWC tensor `X` at
//   th = oh*sh - ph + r*dh,  tw = ow*sw - pw + s*dw
// (after an exact division by divh/divw when those are > 1), zero outside
// [0,IH) x [0,IW).  The forward convolution uses this directly; the
// backward-data pass is the same gather over dY with sh = sw = 1, negated
// padding and tap step, and div = the forward stride.
struct GatherGemm {
    const void* X;          // bf16 (MFMA path) or float32 (fp32 path), NHWC, pixel stride `xs` elements
    const void* Wq;         // packed twn2 codes [NC][wpr]  (or int8 [NC][K] for the int8-stored variant)
    const float* alpha;     // [NC / rows_per_group]
    const float* scale;     // [NC] or null
    const float* shift;     // [NC] or null
    const void* residual;   // like Y or null
    void* Y;                // [M][ldy]
    int64_t M;
    int64_t xs;             // elements between consecutive pixels of X
    int64_t ldy;
    int32_t IH, IW, IC;
    int32_t OH, OW;
    int32_t NC;             // GEMM N (output channels)
    int32_t R, S;
    int32_t sh, sw, ph, pw, dh, dw, divh, divw;
    int32_t K;              // R*S*IC
    int32_t wpr;            // packed words per row
    int32_t rows_per_group;
    int32_t relu;
    int32_t y_f32;          // 1: Y (and residual) float32, 0: bf16
    int32_t plain_gemm;     // 1: R=S=1, stride 1, no padding, OH*OW pixels == rows of X
    int32_t chunk_gather;   // 1: 16-byte chunks are valid although IC/xs are not multiples of 8 (small-C path)
    // Output row remap (strided backward-data as one stride-1 problem per residue class): row m = (n, u, v) of an
    // [N][orU][orV] grid is written to pixel (n, ora + orsh*u, orb + orsw*v) of an [N][orH][orW] image.
    // orU == 0: rows are written in order.
    int32_t orU, orV, orH, orW, ora, orb, orsh, orsw;
    float* partial;         // split-K workspace [splits][M][NC] float32 (float64 on the float32 path; null when splits == 1)
    int32_t splits;         // K is cut into this many ranges of whole 64-wide slabs
};

// Number of K ranges the MFMA path uses for this problem (1 = no split); a pure function of the
// shapes, so the workspace query and the launch agree.
int32_t gather_gemm_splits(const GatherGemm& g);

int32_t launch_gather_gemm_mfma(const GatherGemm& g, int variant, hipStream_t st);

// Small-C first layers (C <= 4, dilation 1): the input is copied once into a zero-bordered
// [N][H+2ph][Wp][4] bf16 tensor so that two horizontally adjacent taps of 4 channels are one
// aligned-enough 16-byte chunk, and the packed codes are re-ordered to k' = (r*Sp + s)*4 + c
// with Sp = S rounded up to even (codes of the phantom tap / channels are zero).
int32_t launch_pad_c4(const uint16_t* X, int N, int H, int W, int C, int ph, int pw, int Hp, int Wp,
                      uint16_t* Xp, hipStream_t st);
// Residue classes of a strided backward-data pass (at most 4: stride products up to 4), by value to the kernel.
struct DxClassTable {
    int32_t count;
    int32_t r0[4], nr[4], s0[4], ns[4], wpr[4];
    int64_t first_word[5];      // offset of each class's codes in the gathered buffer, in 32-bit words
};
int32_t launch_gather_class_codes(const uint32_t* packed_T, int C, int wprT, int S, int O, int sh, int sw,
                                  const DxClassTable& tb, int64_t total_words, uint32_t* out, hipStream_t st);
int32_t launch_zero_fill(void* p, int64_t bytes, hipStream_t st);
int32_t launch_scale_channels(const uint16_t* dY, const float* alpha, int rows_per_group, int O, int64_t pixels,
                              uint16_t* hi, uint16_t* lo, float* one, hipStream_t st);
int32_t launch_pad_repack_c4(const uint16_t* X, int N, int H, int W, int C, int ph, int pw, int Hp, int Wp, uint16_t* Xp,
                             const uint32_t* packed, int rows, int R, int S, int Sp, uint32_t* out, hipStream_t st);
int32_t launch_gather_gemm_dma(const GatherGemm& g, int tile, hipStream_t st);
// Several small unsplit convolution problems of one tile id in one launch of the one-tile-per-workgroup kernel
// (count <= 4); gather_gemm_dma_tile names the tile the dispatcher would use for a problem there (0: none).
int32_t gather_gemm_dma_tile(const GatherGemm& g, bool instead_of_persistent = false);
int32_t launch_gather_gemm_dma_batch(const GatherGemm* gs, int count, int tile, hipStream_t st);
int32_t launch_gather_gemm_fp32(const GatherGemm& g, hipStream_t st);
// K ranges of the float32 path (1 = no split); with more than one, g.partial holds [splits][M][NC] float64 sums.
int32_t gather_gemm_fp32_splits(const GatherGemm& g);
// Multiplication-free comparison kernel (vector ALUs, zero codes skipped); `applicable` is a pure function of the problem.
bool conv_addsub_applicable(const GatherGemm& g);
int32_t launch_conv_addsub(const GatherGemm& g, hipStream_t st);

// Persistent variant of the direct-to-LDS kernel (workgroups walk a list of tiles, loads of the next tile run
// under the epilogue of the last); `applicable` is a pure function of the problem, `tile` one of the ids the
// direct-to-LDS launcher takes (12, 14, 15, 16, 17).
bool conv_stream_applicable(const GatherGemm& g);
int32_t launch_conv_stream(const GatherGemm& g, int tile, hipStream_t st);
int32_t launch_conv_stream_pc(const GatherGemm& g, int tile, int ks, int np, int stages, hipStream_t st);

// 3x3 stride-1 convolutions over 64 input channels (forward, or backward-data with mirrored taps), bf16 in and out,
// output channels a multiple of 64: persistent kernel with the expanded weights resident in registers and the input
// patch of an 8x8 pixel tile (with halo) in LDS; `applicable` is a pure function of the problem.
bool conv_c64_applicable(const GatherGemm& g);
int32_t launch_conv_c64(const GatherGemm& g, hipStream_t st);

// First layers with three input channels, bf16 in and out, dilation 1 (forward): one persistent kernel, no
// workspace and no preparation launch; `applicable` is a pure function of the problem (shapes and alignment).
struct FirstLayer {
    const uint16_t* X;
    const uint32_t* Wq;
    const float* alpha;
    const float* scale;
    const float* shift;
    const uint16_t* residual;
    uint16_t* Y;
    int32_t N, H, W, C, O, R, S, sh, sw, ph, pw, P, Q;
    int32_t rows_per_group, relu;
};
bool conv_first_applicable(const FirstLayer& f);
int32_t launch_conv_first(const FirstLayer& f, hipStream_t st);


// dW[o][c][r][s] = beta*dW + sum_{n,p,q} X[n,ih,iw,c] * dY[n,p,q,o]; dbias[o] = sum dY.
struct WeightGrad {
    const uint16_t* X;      // bf16 NHWC [N][H][W][C]
    const uint16_t* dY;     // bf16 NHWC [N][P][Q][O]
    float* dW;              // [O][C][R][S]
    float* dbias;           // [O] or null
    float* partial;         // workspace: [splits][O][R*S*C] float32
    float beta;
    int32_t N, H, W, C, O, R, S, P, Q;
    int32_t sh, sw, ph, pw, dh, dw;
    int32_t splits;
    // First-layer mode (0 = off): X is the zero-bordered 4-channel copy, a "channel" chunk of 8 is two
    // adjacent taps x 4 channels (C = 8, S = pad_sp/2, dw = 2 above), and the reduction maps
    // j' = (r*pad_sp + s)*4 + c back to [O][c_real][R][s_real], dropping the phantom tap and channels.
    int32_t pad_sp, c_real, s_real;
    int32_t xc;             // elements between consecutive pixels of X (C, or 4 in first-layer mode)
};

// How the weight gradient of one layer is cut up; a pure function of the shapes, shared by the
// workspace query and the launch.
struct WgPlan {
    int32_t patch;          // 1: 128x256 tiles over 32-pixel patches (channel counts multiples of 8); 0: 128x128 tiles over 64 consecutive pixels
    int32_t pn, ph, pw;     // patch = pn images x ph rows x pw columns (pn*ph*pw = 32), powers of two
    int32_t sn, sy, sx;     // patches along batch, rows, columns
    int64_t slabs;          // reduction slabs in total
    int32_t splits;         // blockIdx.y ranges of slabs
    int32_t tiles;          // output tiles (blockIdx.x)
    int32_t ks;             // patch kernel: groups of four waves per workgroup that share a range (1 or 2)
};
WgPlan plan_weight_grad(int32_t N, int32_t P, int32_t Q, int32_t C, int32_t O, int32_t R, int32_t S);
int32_t launch_weight_grad(const WeightGrad& w, hipStream_t st);

}  // namespace twn
