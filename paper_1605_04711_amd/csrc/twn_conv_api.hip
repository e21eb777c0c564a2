// C-ABI entry points of the forward block (Eq. 2; Alg. 1 step 8) and of the
// straight-through backward (Alg. 1 steps 9-10): host-side validation and the
// translation of descriptors into kernel launches.
#include "twn_kernels.h"

using namespace twn;

namespace {

int out_dim(int h, int r, int stride, int pad, int dil) {
    const int64_t eff = static_cast<int64_t>(h) + 2LL * pad - static_cast<int64_t>(dil) * (r - 1) - 1;
    if (eff < 0) return 0;
    return static_cast<int>(eff / stride + 1);
}

int32_t check_conv_desc(const twn_conv_desc* d, int* P, int* Q) {
    if (!d) return TWN_ERR_NULL;
    if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->O <= 0 || d->R <= 0 || d->S <= 0)
        return TWN_ERR_SHAPE;
    if (d->stride_h <= 0 || d->stride_w <= 0 || d->dil_h <= 0 || d->dil_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
        return TWN_ERR_SHAPE;
    if (d->alpha_groups < 1 || d->O % d->alpha_groups != 0) return TWN_ERR_SHAPE;
    *P = out_dim(d->H, d->R, d->stride_h, d->pad_h, d->dil_h);
    *Q = out_dim(d->W, d->S, d->stride_w, d->pad_w, d->dil_w);
    if (*P <= 0 || *Q <= 0) return TWN_ERR_SHAPE;
    const int64_t K = static_cast<int64_t>(d->R) * d->S * d->C;
    const int64_t KT = static_cast<int64_t>(d->R) * d->S * d->O;
    if (K >= (1LL << 30) || KT >= (1LL << 30)) return TWN_ERR_SHAPE;
    if (static_cast<int64_t>(d->N) * d->H * d->W >= (1LL << 31)) return TWN_ERR_SHAPE;
    if (static_cast<int64_t>(d->N) * (*P) * (*Q) >= (1LL << 31)) return TWN_ERR_SHAPE;
    if (d->H >= (1 << 24) || d->W >= (1 << 24)) return TWN_ERR_SHAPE;
    return TWN_OK;
}

int32_t check_dtype(int32_t t) { return (t == TWN_F32 || t == TWN_BF16) ? TWN_OK : TWN_ERR_UNSUPPORTED; }

int32_t check_variant(int32_t variant, int32_t x_dtype) {
    switch (variant) {
        case TWN_VAR_BF16_POSTSCALE: return x_dtype == TWN_BF16 ? TWN_OK : TWN_ERR_UNSUPPORTED;
        case TWN_VAR_FP32: return x_dtype == TWN_F32 ? TWN_OK : TWN_ERR_UNSUPPORTED;
        case TWN_VAR_BF16_ALPHA_LDS:
        case TWN_VAR_I8_STORED_POSTSCALE:
        case TWN_VAR_BF16_SIGN1_POSTSCALE:
        case TWN_VAR_ADDSUB_SPARSE: return x_dtype == TWN_BF16 ? TWN_OK : TWN_ERR_UNSUPPORTED;
        default: return TWN_ERR_UNSUPPORTED;
    }
}

// Output / residual alignment: rows whose channel count and leading dimension are multiples of 8 are written
// with 16-byte stores (and the residual read with 8-byte loads); other shapes are accessed element by element.
int32_t check_out_align(int32_t y_dtype, int64_t NC, int64_t ldy, const void* Y, const void* residual) {
    const size_t elem = (y_dtype == TWN_F32) ? 4 : 2;
    const bool vec = (NC % 8 == 0) && (ldy % 8 == 0);
    if (!aligned(Y, vec ? 16 : elem)) return TWN_ERR_ALIGN;
    if (residual && !aligned(residual, vec ? 16 : elem)) return TWN_ERR_ALIGN;
    return TWN_OK;
}

void set_epilogue(GatherGemm& g, const twn_epilogue* ep) {
    g.scale = ep ? ep->scale : nullptr;
    g.shift = ep ? ep->shift : nullptr;
    g.residual = ep ? ep->residual : nullptr;
    g.relu = ep ? (ep->relu != 0) : 0;
}

size_t splitk_bytes(const GatherGemm& g, int variant) {
    if (variant == TWN_VAR_FP32) {
        const int32_t splits = gather_gemm_fp32_splits(g);
        return splits > 1 ? static_cast<size_t>(splits) * static_cast<size_t>(g.M) * g.NC * sizeof(double) : 0;
    }
    if (variant != TWN_VAR_BF16_POSTSCALE) return 0;   // the other variants never split K
    const int32_t splits = gather_gemm_splits(g);
    return splits > 1 ? static_cast<size_t>(splits) * static_cast<size_t>(g.M) * g.NC * sizeof(float) : 0;
}

// Attaches the split-K workspace (if the problem uses one) and launches.
int32_t dispatch(GatherGemm& g, int variant, void* workspace, size_t workspace_bytes, hipStream_t st,
                 bool allow_split = true) {
    if (variant == TWN_VAR_FP32) {
        g.splits = allow_split ? gather_gemm_fp32_splits(g) : 1;
        g.partial = nullptr;
        if (g.splits > 1) {
            const size_t need = static_cast<size_t>(g.splits) * static_cast<size_t>(g.M) * g.NC * sizeof(double);
            if (!workspace || workspace_bytes < need || !aligned(workspace, 16)) return TWN_ERR_WORKSPACE;
            g.partial = static_cast<float*>(workspace);
        }
        return launch_gather_gemm_fp32(g, st);
    }
    if (variant == TWN_VAR_ADDSUB_SPARSE) {
        g.splits = 1;
        g.partial = nullptr;
        return launch_conv_addsub(g, st);
    }
    if (variant != TWN_VAR_BF16_POSTSCALE) {
        if (variant == TWN_VAR_I8_STORED_POSTSCALE && (g.K % 8 != 0 || !aligned(g.Wq, 8))) return TWN_ERR_UNSUPPORTED;
        if (variant == TWN_VAR_BF16_SIGN1_POSTSCALE) {
            if (!aligned(g.Wq, 16)) return TWN_ERR_ALIGN;
            g.wpr = static_cast<int32_t>(twn_packed1_words_per_row(g.K));    // 1-bit rows
        }
        g.splits = 1;
        g.partial = nullptr;
        return launch_gather_gemm_mfma(g, variant, st);
    }
    g.splits = allow_split ? gather_gemm_splits(g) : 1;
    g.partial = nullptr;
    if (g.splits > 1) {
        const size_t need = static_cast<size_t>(g.splits) * static_cast<size_t>(g.M) * g.NC * sizeof(float);
        if (!workspace || workspace_bytes < need || !aligned(workspace, 16)) return TWN_ERR_WORKSPACE;
        g.partial = static_cast<float*>(workspace);
    }
    return launch_gather_gemm_mfma(g, variant, st);
}

void fill_gemm(GatherGemm& g, const twn_gemm_desc* d) {
    g.M = d->M;
    g.xs = d->ldx ? d->ldx : d->K;
    g.ldy = d->ldy ? d->ldy : d->N;
    g.IH = g.IW = g.OH = g.OW = 1;
    g.IC = d->K;
    g.NC = d->N;
    g.R = g.S = 1;
    g.sh = g.sw = g.dh = g.dw = g.divh = g.divw = 1;
    g.ph = g.pw = 0;
    g.K = d->K;
    g.wpr = static_cast<int32_t>(twn_packed_words_per_row(d->K));
    g.rows_per_group = d->N / d->alpha_groups;
    g.y_f32 = (d->y_dtype == TWN_F32);
    g.plain_gemm = 1;
}

void fill_conv_fwd(GatherGemm& g, const twn_conv_desc* d, int P, int Q) {
    g.M = static_cast<int64_t>(d->N) * P * Q;
    g.xs = d->C;
    g.ldy = d->O;
    g.IH = d->H;
    g.IW = d->W;
    g.IC = d->C;
    g.OH = P;
    g.OW = Q;
    g.NC = d->O;
    g.R = d->R;
    g.S = d->S;
    g.sh = d->stride_h;
    g.sw = d->stride_w;
    g.ph = d->pad_h;
    g.pw = d->pad_w;
    g.dh = d->dil_h;
    g.dw = d->dil_w;
    g.divh = g.divw = 1;
    g.K = d->R * d->S * d->C;
    g.wpr = static_cast<int32_t>(twn_packed_words_per_row(g.K));
    g.rows_per_group = d->O / d->alpha_groups;
    g.y_f32 = (d->y_dtype == TWN_F32);
    g.plain_gemm = (d->R == 1 && d->S == 1 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 0 &&
                    d->pad_w == 0);
}

// dX = gather over dY: row (n,h,w), k = (r,s,o):
//   p = (h + ph - r*dh)/sh when divisible, q likewise; weights = transposed packed copy.
void fill_conv_bwd_data(GatherGemm& g, const twn_conv_desc* d, int P, int Q) {
    g.M = static_cast<int64_t>(d->N) * d->H * d->W;
    g.xs = d->O;
    g.ldy = d->C;
    g.IH = P;
    g.IW = Q;
    g.IC = d->O;
    g.OH = d->H;
    g.OW = d->W;
    g.NC = d->C;
    g.R = d->R;
    g.S = d->S;
    g.sh = g.sw = 1;
    g.ph = -d->pad_h;
    g.pw = -d->pad_w;
    g.dh = -d->dil_h;
    g.dw = -d->dil_w;
    g.divh = d->stride_h;
    g.divw = d->stride_w;
    g.K = d->R * d->S * d->O;
    g.wpr = static_cast<int32_t>(twn_packed_words_per_row(g.K));
    g.rows_per_group = d->C;
    g.y_f32 = (d->y_dtype == TWN_F32);
    g.plain_gemm = (d->R == 1 && d->S == 1 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 0 &&
                    d->pad_w == 0);
}

// ---- small-C forward path (C <= 4, bf16, dilation 1): geometry of the padded copy ----
struct SmallC {
    int Hp, Wp, Sp;
    size_t x_bytes, w_bytes;
};

bool small_c(const twn_conv_desc* d, SmallC* sc) {
    if (d->variant != TWN_VAR_BF16_POSTSCALE || d->x_dtype != TWN_BF16) return false;
    if (d->C > 4 || d->dil_h != 1 || d->dil_w != 1) return false;
    sc->Sp = (d->S + 1) & ~1;
    sc->Hp = d->H + 2 * d->pad_h;
    sc->Wp = d->W + 2 * d->pad_w + (sc->Sp - d->S);
    sc->x_bytes = round_up(static_cast<size_t>(d->N) * sc->Hp * sc->Wp * 4 * sizeof(uint16_t), 256);
    sc->w_bytes = round_up(twn_packed_bytes(d->O, static_cast<int64_t>(d->R) * sc->Sp * 4), 256);
    return static_cast<int64_t>(d->N) * sc->Hp * sc->Wp < (1LL << 31);
}

void fill_conv_fwd_small_c(GatherGemm& g, const twn_conv_desc* d, const SmallC& sc, int P, int Q) {
    fill_conv_fwd(g, d, P, Q);
    g.xs = 4;                    // elements per padded pixel
    g.IH = sc.Hp;
    g.IW = sc.Wp;
    g.IC = 8;                    // one 16-byte chunk = two adjacent taps x 4 channels
    g.S = sc.Sp / 2;
    g.ph = g.pw = 0;             // the border is part of the copy
    g.dw = 2;                    // chunk j of a filter row starts 2 pixels after chunk j-1
    g.K = d->R * sc.Sp * 4;
    g.wpr = static_cast<int32_t>(twn_packed_words_per_row(g.K));
    g.plain_gemm = 0;
    g.chunk_gather = 1;
}

// Strided backward-data as stride-1 problems, one per residue class (a, b) of the output pixels
// (h = a + sh*u, w = b + sw*v): the taps that reach the class are r = r0 + jr*sh with r0 = (a + pad_h) % sh, the
// coordinate read is p = u + (a + pad_h - r0)/sh - jr, i.e. an undivided gather with dilation -1.  Used for
// dilation 1, O % 64 == 0 (every tap is whole K slabs), C % 8 == 0, stride products up to 4.
struct DxClasses {
    int count;                  // classes that have taps
    bool any_empty;             // some class has none: those pixels of dX are zero
    GatherGemm g[4];
    DxClassTable tb;
    int64_t code_words;
};

bool strided_dx_classes(const twn_conv_desc* d, int P, int Q, DxClasses* out) {
    const int sh = d->stride_h, sw = d->stride_w;
    if (sh * sw <= 1 || sh * sw > 4 || d->dil_h != 1 || d->dil_w != 1 || d->O % 64 != 0 || d->C % 8 != 0 ||
        d->variant != TWN_VAR_BF16_POSTSCALE || d->x_dtype != TWN_BF16)
        return false;
    // several small launches only pay when each class still has enough pixels to fill the chip
    if (static_cast<int64_t>(d->N) * ((d->H + sh - 1) / sh) * ((d->W + sw - 1) / sw) < env_int("TWN_DX_CLASS_MIN_PIXELS", 2048))
        return false;
    out->count = 0;
    out->any_empty = false;
    out->code_words = 0;
    for (int a = 0; a < sh; ++a)
        for (int b = 0; b < sw; ++b) {
            const int U = (d->H - a + sh - 1) / sh, V = (d->W - b + sw - 1) / sw;
            if (U <= 0 || V <= 0) continue;         // no pixel in this class
            const int r0 = (a + d->pad_h) % sh, s0 = (b + d->pad_w) % sw;
            const int nr = r0 < d->R ? (d->R - r0 + sh - 1) / sh : 0, ns = s0 < d->S ? (d->S - s0 + sw - 1) / sw : 0;
            if (nr == 0 || ns == 0) {
                out->any_empty = true;
                continue;
            }
            const int k = out->count++;
            GatherGemm& g = out->g[k];
            g = GatherGemm{};
            fill_conv_bwd_data(g, d, P, Q);
            g.M = static_cast<int64_t>(d->N) * U * V;
            g.OH = U;
            g.OW = V;
            g.R = nr;
            g.S = ns;
            g.ph = -((a + d->pad_h - r0) / sh);
            g.pw = -((b + d->pad_w - s0) / sw);
            g.dh = g.dw = -1;
            g.divh = g.divw = 1;
            g.K = nr * ns * d->O;
            g.wpr = static_cast<int32_t>(twn_packed_words_per_row(g.K));
            g.plain_gemm = 0;
            g.orU = U; g.orV = V; g.orH = d->H; g.orW = d->W;
            g.ora = a; g.orb = b; g.orsh = sh; g.orsw = sw;
            out->tb.r0[k] = r0; out->tb.nr[k] = nr; out->tb.s0[k] = s0; out->tb.ns[k] = ns;
            out->tb.wpr[k] = g.wpr;
            out->tb.first_word[k] = out->code_words;
            out->code_words += static_cast<int64_t>(d->C) * g.wpr;
        }
    out->tb.count = out->count;
    for (int k = out->count; k <= 4; ++k) out->tb.first_word[k] = out->code_words;
    return out->count > 0;
}

size_t scaled_dy_bytes(const twn_conv_desc* d, int P, int Q);
size_t scaled_dy_term_bytes(const twn_conv_desc* d, int P, int Q);

// Workspace of the class path: gathered codes (256-byte multiple) + the two scaled copies of dY (several alphas
// only) + the largest split-K need of a class.
size_t strided_dx_bytes(const twn_conv_desc* d, int P, int Q) {
    DxClasses cl;
    if (!strided_dx_classes(d, P, Q, &cl)) return 0;
    size_t split = 0;
    for (int k = 0; k < cl.count; ++k) {
        const size_t b = splitk_bytes(cl.g[k], d->variant);
        if (b > split) split = b;
    }
    return round_up(static_cast<size_t>(cl.code_words) * sizeof(uint32_t), 256) + scaled_dy_bytes(d, P, Q) + split;
}

// Backward-data with one alpha per group of filters: two scaled copies of dY (high and low bf16 term) + one float
// (the unit alpha).
size_t scaled_dy_term_bytes(const twn_conv_desc* d, int P, int Q) {
    return round_up(static_cast<size_t>(d->N) * P * Q * d->O * sizeof(uint16_t), 256);
}
size_t scaled_dy_bytes(const twn_conv_desc* d, int P, int Q) {
    if (d->alpha_groups == 1) return 0;
    return 2 * scaled_dy_term_bytes(d, P, Q) + 256;
}

// Weight-gradient workspace: [padded copy of X in first-layer mode] + split partials + bias partials.
size_t weight_grad_bytes(const twn_conv_desc* d, int P, int Q) {
    SmallC sc;
    if (small_c(d, &sc) && d->O % 8 == 0) {
        const int64_t Jp = static_cast<int64_t>(d->R) * sc.Sp * 4;
        const int64_t splits = plan_weight_grad(d->N, P, Q, 8, d->O, d->R, sc.Sp / 2).splits;
        return sc.x_bytes + static_cast<size_t>((splits * d->O * Jp + 64LL * d->O) * sizeof(float));
    }
    const int64_t J = static_cast<int64_t>(d->R) * d->S * d->C;
    const int64_t splits = plan_weight_grad(d->N, P, Q, d->C, d->O, d->R, d->S).splits;
    return static_cast<size_t>((splits * d->O * J + 64LL * d->O) * sizeof(float));
}

}  // namespace

extern "C" size_t twn_gemm_fwd_workspace_bytes(const twn_gemm_desc* d) {
    if (!d || d->M <= 0 || d->N <= 0 || d->K <= 0 || d->alpha_groups < 1) return 0;
    GatherGemm g{};
    fill_gemm(g, d);
    return splitk_bytes(g, d->variant);
}

extern "C" int32_t twn_gemm_fwd(const twn_gemm_desc* d, const void* X, const void* weights,
                                const float* alpha, const twn_epilogue* ep, void* Y,
                                void* workspace, size_t workspace_bytes, void* stream) {
    if (!d || !X || !weights || !alpha || !Y) return TWN_ERR_NULL;
    if (d->M <= 0 || d->N <= 0 || d->K <= 0 || d->M >= (1LL << 31) || d->K >= (1 << 30)) return TWN_ERR_SHAPE;
    if (d->alpha_groups < 1 || d->N % d->alpha_groups != 0) return TWN_ERR_SHAPE;
    int32_t rc = check_dtype(d->x_dtype);
    if (rc == TWN_OK) rc = check_dtype(d->y_dtype);
    if (rc == TWN_OK) rc = check_variant(d->variant, d->x_dtype);
    if (rc != TWN_OK) return rc;
    const int64_t ldx = d->ldx ? d->ldx : d->K;
    const int64_t ldy = d->ldy ? d->ldy : d->N;
    if (ldx < d->K || ldy < d->N) return TWN_ERR_SHAPE;
    if (!aligned(weights, 16)) return TWN_ERR_ALIGN;
    if (d->x_dtype == TWN_BF16 && !aligned(X, 2)) return TWN_ERR_ALIGN;
    if (d->x_dtype == TWN_F32 && !aligned(X, 4)) return TWN_ERR_ALIGN;
    if (d->x_dtype == TWN_BF16 && d->K % 8 == 0 && ldx % 8 == 0 && !aligned(X, 16)) return TWN_ERR_ALIGN;
    rc = check_out_align(d->y_dtype, d->N, ldy, Y, ep ? ep->residual : nullptr);
    if (rc != TWN_OK) return rc;

    GatherGemm g{};
    g.X = X;
    g.Wq = weights;
    g.alpha = alpha;
    set_epilogue(g, ep);
    g.Y = Y;
    fill_gemm(g, d);
    return dispatch(g, d->variant, workspace, workspace_bytes, as_stream(stream));
}

extern "C" size_t twn_conv2d_fwd_workspace_bytes(const twn_conv_desc* d) {
    int P, Q;
    if (check_conv_desc(d, &P, &Q) != TWN_OK) return 0;
    GatherGemm g{};
    SmallC sc;
    if (small_c(d, &sc)) {
        fill_conv_fwd_small_c(g, d, sc, P, Q);
        return sc.x_bytes + sc.w_bytes + splitk_bytes(g, d->variant);
    }
    fill_conv_fwd(g, d, P, Q);
    return splitk_bytes(g, d->variant);
}

extern "C" int32_t twn_conv2d_fwd(const twn_conv_desc* d, const void* X, const void* weights,
                                  const float* alpha, const twn_epilogue* ep, void* Y,
                                  void* workspace, size_t workspace_bytes, void* stream) {
    int P, Q;
    int32_t rc = check_conv_desc(d, &P, &Q);
    if (rc != TWN_OK) return rc;
    if (!X || !weights || !alpha || !Y) return TWN_ERR_NULL;
    rc = check_dtype(d->x_dtype);
    if (rc == TWN_OK) rc = check_dtype(d->y_dtype);
    if (rc == TWN_OK) rc = check_variant(d->variant, d->x_dtype);
    if (rc != TWN_OK) return rc;
    if (!aligned(weights, 16)) return TWN_ERR_ALIGN;
    if (d->x_dtype == TWN_BF16 && !aligned(X, (d->C % 8 == 0) ? 16 : 2)) return TWN_ERR_ALIGN;
    if (d->x_dtype == TWN_F32 && !aligned(X, 4)) return TWN_ERR_ALIGN;
    rc = check_out_align(d->y_dtype, d->O, d->O, Y, ep ? ep->residual : nullptr);
    if (rc != TWN_OK) return rc;

    GatherGemm g{};
    g.X = X;
    g.Wq = weights;
    g.alpha = alpha;
    set_epilogue(g, ep);
    g.Y = Y;
    if (d->variant == TWN_VAR_BF16_POSTSCALE && d->x_dtype == TWN_BF16 && d->y_dtype == TWN_BF16 && d->C == 3 &&
        d->dil_h == 1 && d->dil_w == 1 && env_int("TWN_FIRST", 1) != 0) {
        // three-channel first layer: persistent kernel with the input patch widened to four channels in LDS and
        // the expanded weights resident in registers (no workspace, no preparation launch)
        FirstLayer f{};
        f.X = static_cast<const uint16_t*>(X);
        f.Wq = static_cast<const uint32_t*>(weights);
        f.alpha = alpha;
        f.scale = g.scale;
        f.shift = g.shift;
        f.residual = static_cast<const uint16_t*>(g.residual);
        f.Y = static_cast<uint16_t*>(Y);
        f.N = d->N; f.H = d->H; f.W = d->W; f.C = d->C; f.O = d->O; f.R = d->R; f.S = d->S;
        f.sh = d->stride_h; f.sw = d->stride_w; f.ph = d->pad_h; f.pw = d->pad_w; f.P = P; f.Q = Q;
        f.rows_per_group = d->O / d->alpha_groups;
        f.relu = g.relu;
        if (conv_first_applicable(f)) return launch_conv_first(f, as_stream(stream));
    }
    SmallC sc;
    if (small_c(d, &sc)) {
        // first-layer path: padded 4-channel copy of X and re-ordered codes live in the workspace
        fill_conv_fwd_small_c(g, d, sc, P, Q);
        const size_t head = sc.x_bytes + sc.w_bytes;
        if (!workspace || workspace_bytes < head + splitk_bytes(g, d->variant) || !aligned(workspace, 256))
            return TWN_ERR_WORKSPACE;
        hipStream_t st = as_stream(stream);
        uint16_t* Xp = static_cast<uint16_t*>(workspace);
        uint32_t* Wp = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(workspace) + sc.x_bytes);
        rc = launch_pad_repack_c4(static_cast<const uint16_t*>(X), d->N, d->H, d->W, d->C, d->pad_h, d->pad_w, sc.Hp,
                                  sc.Wp, Xp, static_cast<const uint32_t*>(weights), d->O, d->R, d->S, sc.Sp, Wp, st);
        if (rc != TWN_OK) return rc;
        g.X = Xp;
        g.Wq = Wp;
        return dispatch(g, d->variant, static_cast<unsigned char*>(workspace) + head, workspace_bytes - head, st);
    }
    fill_conv_fwd(g, d, P, Q);
    return dispatch(g, d->variant, workspace, workspace_bytes, as_stream(stream));
}

// One problem of twn_conv2d_fwd_pair: the checks of twn_conv2d_fwd for the product variant on bf16 tensors whose
// channel count is a multiple of 8 (no first-layer paths), then the problem descriptor.
static int32_t build_pair_problem(const twn_conv_desc* d, const void* X, const void* weights, const float* alpha,
                                  const twn_epilogue* ep, void* Y, GatherGemm* g) {
    int P, Q;
    int32_t rc = check_conv_desc(d, &P, &Q);
    if (rc != TWN_OK) return rc;
    if (!X || !weights || !alpha || !Y) return TWN_ERR_NULL;
    if (d->variant != TWN_VAR_BF16_POSTSCALE || d->x_dtype != TWN_BF16 || d->y_dtype != TWN_BF16 || d->C % 8 != 0)
        return TWN_ERR_UNSUPPORTED;
    if (!aligned(weights, 16) || !aligned(X, 16)) return TWN_ERR_ALIGN;
    rc = check_out_align(d->y_dtype, d->O, d->O, Y, ep ? ep->residual : nullptr);
    if (rc != TWN_OK) return rc;
    *g = GatherGemm{};
    g->X = X;
    g->Wq = weights;
    g->alpha = alpha;
    set_epilogue(*g, ep);
    g->Y = Y;
    fill_conv_fwd(*g, d, P, Q);
    g->splits = 1;
    g->partial = nullptr;
    return TWN_OK;
}

extern "C" int32_t twn_conv2d_fwd_pair(const twn_conv_desc* d0, const twn_conv_desc* d1, const void* X,
                                       const void* weights0, const float* alpha0, const twn_epilogue* ep0, void* Y0,
                                       const void* weights1, const float* alpha1, const twn_epilogue* ep1, void* Y1,
                                       void* stream) {
    if (!d0 || !d1) return TWN_ERR_NULL;
    if (d0->N != d1->N || d0->H != d1->H || d0->W != d1->W || d0->C != d1->C) return TWN_ERR_SHAPE;
    GatherGemm g[2];
    int32_t rc = build_pair_problem(d0, X, weights0, alpha0, ep0, Y0, &g[0]);
    if (rc == TWN_OK) rc = build_pair_problem(d1, X, weights1, alpha1, ep1, Y1, &g[1]);
    if (rc != TWN_OK) return rc;
    hipStream_t st = as_stream(stream);
    const int t0 = gather_gemm_dma_tile(g[0], true), t1 = gather_gemm_dma_tile(g[1], true);
    // One launch pays while the reduction is short: with more than 24 slabs per tile the persistent kernels with load
    // waves win back more than the saved launch (ResNet-18 b64 block heads, two launches -> one: 128 filters, K = 576:
    // 23.4 -> 19.1 us; 256 filters, K = 1152: 17.9 -> 15.9 us; 512 filters, K = 2304: 18.2 -> 19.3 us).
    const int64_t kmax = g[0].K > g[1].K ? g[0].K : g[1].K;
    const int pair_knob = env_int("TWN_FWD_PAIR", 1);          // 0: never one launch, 2: whenever the tiles agree
    if (t0 != 0 && t0 == t1 && (pair_knob == 2 || (pair_knob == 1 && kmax <= 1536))) {
        rc = launch_gather_gemm_dma_batch(g, 2, t0, st);
        if (rc != TWN_ERR_UNSUPPORTED) return rc;
    }
    // different tile shapes (or no build for the pair): one after the other, as two twn_conv2d_fwd calls without a workspace
    rc = dispatch(g[0], d0->variant, nullptr, 0, st, false);
    if (rc != TWN_OK) return rc;
    return dispatch(g[1], d1->variant, nullptr, 0, st, false);
}

extern "C" size_t twn_conv2d_bwd_ste_workspace_bytes(const twn_conv_desc* d) {
    int P, Q;
    if (check_conv_desc(d, &P, &Q) != TWN_OK) return 0;
    // the data-gradient split-K partials and the weight-gradient partials use the workspace one after the other
    GatherGemm g{};
    fill_conv_bwd_data(g, d, P, Q);
    size_t a = scaled_dy_bytes(d, P, Q) + splitk_bytes(g, d->variant);
    const size_t a2 = strided_dx_bytes(d, P, Q);
    if (a2 > a) a = a2;
    const size_t b = weight_grad_bytes(d, P, Q);
    return a > b ? a : b;
}

extern "C" int32_t twn_conv2d_bwd_ste(const twn_conv_desc* d, const void* X, const void* dY,
                                      const uint32_t* packed_T, const float* alpha,
                                      void* dX, float* dW, float* dbias, float dW_beta,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    int P, Q;
    int32_t rc = check_conv_desc(d, &P, &Q);
    if (rc != TWN_OK) return rc;
    if (!dY) return TWN_ERR_NULL;
    if (dX && (!packed_T || !alpha)) return TWN_ERR_NULL;
    if (dW && !X) return TWN_ERR_NULL;
    // the int8-stored comparison variant is forward-only: the transposed codes of this call are 2-bit packed
    if (d->x_dtype != TWN_BF16 ||
        (d->variant != TWN_VAR_BF16_POSTSCALE && d->variant != TWN_VAR_BF16_ALPHA_LDS)) return TWN_ERR_UNSUPPORTED;
    rc = check_dtype(d->y_dtype);
    if (rc != TWN_OK) return rc;
    if (dW_beta != 0.0f && dW_beta != 1.0f) return TWN_ERR_UNSUPPORTED;
    if (!aligned(dY, (d->O % 8 == 0) ? 16 : 2)) return TWN_ERR_ALIGN;
    if (X && !aligned(X, (d->C % 8 == 0) ? 16 : 2)) return TWN_ERR_ALIGN;
    if (packed_T && !aligned(packed_T, 16)) return TWN_ERR_ALIGN;
    if (dW && !aligned(dW, 4)) return TWN_ERR_ALIGN;
    if (dX) {
        rc = check_out_align(d->y_dtype, d->C, d->C, dX, nullptr);
        if (rc != TWN_OK) return rc;
    }
    if (dW || dbias) {
        const size_t need = weight_grad_bytes(d, P, Q);
        if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) return TWN_ERR_WORKSPACE;
    }
    hipStream_t st = as_stream(stream);

    DxClasses cl;
    if (dX && env_int("TWN_DX_CLASSES", 1) != 0 && strided_dx_classes(d, P, Q, &cl) && workspace &&
        workspace_bytes >= strided_dx_bytes(d, P, Q) && aligned(workspace, 256) && aligned(dX, 16)) {
        // strided layer: one stride-1 contraction per residue class of the output pixels
        const size_t code_bytes = round_up(static_cast<size_t>(cl.code_words) * sizeof(uint32_t), 256);
        uint32_t* codes = static_cast<uint32_t*>(workspace);
        rc = launch_gather_class_codes(packed_T, d->C, static_cast<int>(twn_packed_words_per_row(
                                           static_cast<int64_t>(d->R) * d->S * d->O)),
                                       d->S, d->O, d->stride_h, d->stride_w, cl.tb, cl.code_words, codes, st);
        if (rc != TWN_OK) return rc;
        if (cl.any_empty) {
            const int64_t bytes = static_cast<int64_t>(d->N) * d->H * d->W * d->C * (d->y_dtype == TWN_F32 ? 4 : 2);
            rc = launch_zero_fill(dX, bytes, st);
            if (rc != TWN_OK) return rc;
        }
        // several alphas: the two bf16 terms of alpha_o * dY, as in the undivided path below
        const size_t head = scaled_dy_bytes(d, P, Q);
        unsigned char* wsb = static_cast<unsigned char*>(workspace) + code_bytes;
        const uint16_t* hi = nullptr;
        const uint16_t* lo = nullptr;
        const float* one = nullptr;
        if (head) {
            uint16_t* h = reinterpret_cast<uint16_t*>(wsb);
            uint16_t* l = reinterpret_cast<uint16_t*>(wsb + scaled_dy_term_bytes(d, P, Q));
            float* o1 = reinterpret_cast<float*>(wsb + head - 256);
            rc = launch_scale_channels(static_cast<const uint16_t*>(dY), alpha, d->O / d->alpha_groups, d->O,
                                       static_cast<int64_t>(d->N) * P * Q, h, l, o1, st);
            if (rc != TWN_OK) return rc;
            hi = h; lo = l; one = o1;
        }
        for (int k = 0; k < cl.count; ++k) {
            GatherGemm& g = cl.g[k];
            g.X = head ? static_cast<const void*>(hi) : dY;
            g.Wq = codes + cl.tb.first_word[k];
            g.alpha = head ? one : alpha;
            g.Y = dX;
            g.splits = 1;
            g.partial = nullptr;
        }
        // all classes in ONE launch when the dispatcher would give each of them the same tile of the
        // one-tile-per-workgroup kernel (they are too small to be worth a launch each: ResNet-18 b64, the three
        // strided 3x3 layers 33 / 34 / 48 us as four launches)
        int batch_tile = env_int("TWN_DX_CLASS_BATCH", 1) != 0 ? gather_gemm_dma_tile(cl.g[0]) : 0;
        for (int k = 1; k < cl.count && batch_tile; ++k)
            if (gather_gemm_dma_tile(cl.g[k]) != batch_tile) batch_tile = 0;
        if (batch_tile && cl.count > 1 && d->variant == TWN_VAR_BF16_POSTSCALE) {
            rc = launch_gather_gemm_dma_batch(cl.g, cl.count, batch_tile, st);
            if (rc == TWN_OK && head) {
                for (int k = 0; k < cl.count; ++k) {
                    cl.g[k].X = lo;
                    cl.g[k].residual = dX;
                }
                rc = launch_gather_gemm_dma_batch(cl.g, cl.count, batch_tile, st);
            }
            if (rc != TWN_ERR_UNSUPPORTED) {
                if (rc != TWN_OK) return rc;
                cl.count = 0;       // done
            } else {
                for (int k = 0; k < cl.count; ++k) {
                    cl.g[k].X = head ? static_cast<const void*>(hi) : dY;
                    cl.g[k].residual = nullptr;
                }
            }
        }
        for (int k = 0; k < cl.count; ++k) {
            GatherGemm& g = cl.g[k];
            // no split-K here: a class is one of several launches of a layer whose own launch would not be split either,
            // and partial tiles plus a finishing launch per class cost more than the idle CUs (ResNet-18 stage 4: 70 -> 48 us)
            rc = dispatch(g, d->variant, wsb + head, workspace_bytes - code_bytes - head, st, false);
            if (rc != TWN_OK) return rc;
            if (head) {
                g.X = lo;
                g.residual = dX;
                rc = dispatch(g, d->variant, wsb + head, workspace_bytes - code_bytes - head, st, false);
                if (rc != TWN_OK) return rc;
            }
        }
    } else if (dX) {
        GatherGemm g{};
        g.X = dY;
        g.Wq = packed_T;
        g.alpha = alpha;
        g.Y = dX;
        fill_conv_bwd_data(g, d, P, Q);
        unsigned char* ws = static_cast<unsigned char*>(workspace);
        size_t ws_bytes = workspace_bytes;
        const size_t head = scaled_dy_bytes(d, P, Q);
        if (head) {
            // alpha multiplies per forward output channel o, which is a K index here: with several alphas dY is
            // scaled first (into the workspace) and the contraction runs with alpha = 1
            if (!workspace || workspace_bytes < head + splitk_bytes(g, d->variant) || !aligned(workspace, 256))
                return TWN_ERR_WORKSPACE;
            uint16_t* hi = static_cast<uint16_t*>(workspace);
            uint16_t* lo = reinterpret_cast<uint16_t*>(ws + scaled_dy_term_bytes(d, P, Q));
            float* one = reinterpret_cast<float*>(ws + head - 256);
            rc = launch_scale_channels(static_cast<const uint16_t*>(dY), alpha, d->O / d->alpha_groups, d->O,
                                       static_cast<int64_t>(d->N) * P * Q, hi, lo, one, st);
            if (rc != TWN_OK) return rc;
            g.X = hi;
            g.alpha = one;
            ws += head;
            ws_bytes -= head;
            rc = dispatch(g, d->variant, ws, ws_bytes, st);
            if (rc != TWN_OK) return rc;
            // second term, added onto the first: every output element is read (as the residual) and written by the
            // same thread of the second pass
            g.X = lo;
            g.residual = dX;
        }
        rc = dispatch(g, d->variant, ws, ws_bytes, st);
        if (rc != TWN_OK) return rc;
    }
    if (dW || dbias) {
        WeightGrad w{};
        w.X = static_cast<const uint16_t*>(X);
        w.dY = static_cast<const uint16_t*>(dY);
        w.dW = dW;
        w.dbias = dbias;
        w.partial = static_cast<float*>(workspace);
        w.beta = dW_beta;
        w.N = d->N; w.H = d->H; w.W = d->W; w.C = d->C; w.O = d->O; w.R = d->R; w.S = d->S;
        w.P = P; w.Q = Q;
        w.sh = d->stride_h; w.sw = d->stride_w; w.ph = d->pad_h; w.pw = d->pad_w;
        w.dh = d->dil_h; w.dw = d->dil_w;
        w.xc = d->C;
        SmallC sc;
        if (dW && small_c(d, &sc) && d->O % 8 == 0) {
            // first-layer mode: gather from the zero-bordered 4-channel copy (rebuilt here: the call is stateless)
            uint16_t* Xp = static_cast<uint16_t*>(workspace);
            rc = launch_pad_c4(static_cast<const uint16_t*>(X), d->N, d->H, d->W, d->C, d->pad_h, d->pad_w, sc.Hp,
                               sc.Wp, Xp, st);
            if (rc != TWN_OK) return rc;
            w.X = Xp;
            w.partial = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + sc.x_bytes);
            w.H = sc.Hp; w.W = sc.Wp; w.C = 8; w.S = sc.Sp / 2;
            w.ph = w.pw = 0; w.dw = 2;
            w.xc = 4;
            w.pad_sp = sc.Sp; w.c_real = d->C; w.s_real = d->S;
        }
        w.splits = plan_weight_grad(d->N, P, Q, w.C, d->O, d->R, w.S).splits;
        rc = launch_weight_grad(w, st);
    }
    return rc;
}
