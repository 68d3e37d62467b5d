// TrainClient (Alg. 1) / the inner loop of Alg. 3: forward, backward and AdamW for the
// decoder-only transformer of Table 4, as a fixed sequence of kernel launches on one stream.
//
// Per block:  a = LN(x; g1); qkv = a Wqkv; o = CausalALiBiAttention(qkv); x' = x + o Wo;
//             b = LN(x'; g2); h = b W1; u = GELU(h); x'' = x' + u W2   (GELU'(h) is saved, not h).
// Head:       y = LN(x; gf); z = y E^T (tied); loss = mean(logsumexp(z) - z_target).
// The LM head is walked in row chunks so that only [chunk, vocab] logits exist at a time:
// logits -> in-place softmax-minus-onehot -> dy and dE GEMMs.

#include <cmath>
#include <new>
#include <vector>

#include "kernels.h"

namespace {

struct Layout {
    int64_t E = 0, gf = 0, total = 0;
    std::vector<int64_t> g1, wqkv, wo, g2, w1, w2;
};

Layout make_layout(const photon_model_cfg &c) {
    Layout l;
    const int64_t d = c.d_model, f = c.d_ff;
    int64_t pos = (int64_t)c.vocab * d;
    for (int i = 0; i < c.n_layers; ++i) {
        l.g1.push_back(pos); pos += d;
        l.wqkv.push_back(pos); pos += 3 * d * d;
        l.wo.push_back(pos); pos += d * d;
        l.g2.push_back(pos); pos += d;
        l.w1.push_back(pos); pos += d * f;
        l.w2.push_back(pos); pos += f * d;
    }
    l.gf = pos;
    l.total = pos + d;
    return l;
}

// activations one block keeps for its backward pass
struct BlockActs {
    void *a = nullptr, *qkv = nullptr, *o = nullptr, *b = nullptr, *h = nullptr, *u = nullptr;  // T
    float *x_mid = nullptr, *mean1 = nullptr, *rstd1 = nullptr, *mean2 = nullptr, *rstd2 = nullptr, *lse = nullptr;
};

}  // namespace

struct ModelWorkspace {
    Layout lay;
    int M = 0, chunk = 0, ldz = 0;
    size_t tsize = 4;
    std::vector<void *> allocs;
    bf16 *w16 = nullptr;         // bf16 working copy of the parameters (bf16 mode)
    bf16 *w16t = nullptr;        // the same matrices transposed ([out, in]): forward products read both
                                 // operands K-contiguous
    float *grads = nullptr;      // fp32 gradient accumulators [N]
    std::vector<float *> x_in;   // [L + 1] residual stream at every block boundary
    std::vector<BlockActs> acts; // L slots, or 1 when blocks are recomputed
    float *meanf = nullptr, *rstdf = nullptr;
    void *y = nullptr, *logits = nullptr;
    float *loss_rows = nullptr;
    double *loss_acc = nullptr;  // device, one per step
    int *tok_flag = nullptr;     // device: set by the token-id range check
    int loss_cap = 0;
    // backward temporaries
    float *dx_a = nullptr, *dx_b = nullptr, *dvec = nullptr, *ln_scratch = nullptr;
    void *dx16 = nullptr, *dff = nullptr, *dqkv = nullptr, *dtmp = nullptr, *dy = nullptr;
    float *splitk = nullptr;
    size_t splitk_bytes = 0;
    void *adam_table = nullptr;  // device table of the vector's matrices for the tiled AdamW (bf16 mode)
    int adam_mats = 0, adam_tiles = 0;
};

namespace {

template <typename P>
int dev_alloc(photon_ctx *ctx, P **out, size_t bytes) {
    void *p = nullptr;
    const hipError_t e = hipMalloc(&p, bytes ? bytes : 16);
    if (e != hipSuccess) {
        ctx->last_hip_error = (int)e;
        return PHOTON_ENOMEM;
    }
    ctx->ws->allocs.push_back(p);
    ctx->workspace_bytes += (int64_t)bytes;
    *out = reinterpret_cast<P *>(p);
    return PHOTON_OK;
}

#define TRY_RC(expr)                    \
    do {                                \
        const int rc_ = (expr);         \
        if (rc_ != PHOTON_OK) return rc_; \
    } while (0)

// ---------------------------------------------------------------------------------------------

template <typename T>
struct Runner {
    photon_ctx *ctx;
    ModelWorkspace &w;
    const photon_model_cfg &c;
    hipStream_t st;
    const float *params;  // fp32 masters (gains, embedding gather)
    const T *wmat;        // matmul operands: params (fp32 mode) or the bf16 copy
    const T *wmat_t;      // transposed matrices (bf16 mode only)
    float *grads;
    float beta = 1.f;     // 0 on the first pass of an optimizer step: gradients are overwritten, not
                          // accumulated, so the accumulators need no clearing pass (and no read)
    int Bm, S, d, F, V, H, Dh, M;

    // batch: sequences per pass (the ctx micro-batch, or several of them fused)
    Runner(photon_ctx *cx, const float *p, float *g, int batch)
        : ctx(cx), w(*cx->ws), c(cx->cfg), st(cx->stream), params(p), grads(g) {
        gemm_set_splitk_workspace(w.splitk, w.splitk_bytes);
        Bm = batch; S = c.seq_len; d = c.d_model; F = c.d_ff; V = c.vocab; H = c.n_heads;
        Dh = d / H; M = Bm * S;
        if constexpr (sizeof(T) == 2) {
            wmat = reinterpret_cast<const T *>(w.w16);
            wmat_t = reinterpret_cast<const T *>(w.w16t);
        } else {
            wmat = reinterpret_cast<const T *>(p);
            wmat_t = nullptr;
        }
    }

    // C = A W for a weight W [K, N] at offset woff of the flat vector: bf16 mode multiplies by
    // the transposed copy (both operands K-contiguous), fp32 mode by W itself.
    void gemm_w(GemmEpi epi, GemmArgs g, int64_t woff) {
        if (wmat_t) {
            g.B = wmat_t + woff;
            g.ldb = g.K;
            gemm<T>(st, GEMM_NT, epi, g);
        } else {
            g.B = wmat + woff;
            g.ldb = g.N;
            gemm<T>(st, GEMM_NN, epi, g);
        }
    }

    static GemmArgs ga(int M_, int N_, int K_, const void *A, int lda, const void *B, int ldb, void *C, int ldc) {
        GemmArgs g;
        g.M = M_; g.N = N_; g.K = K_; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
        return g;
    }

    void block_forward(int l, const float *x_in, BlockActs &a, float *x_out) {
        const Layout &L = w.lay;
        layernorm_fwd<T>(st, x_in, params + L.g1[l], (T *)a.a, a.mean1, a.rstd1, M, d, c.ln_eps);
        gemm_w(EPI_STORE, ga(M, 3 * d, d, a.a, d, nullptr, 0, a.qkv, 3 * d), L.wqkv[l]);
        attention_fwd<T>(st, (const T *)a.qkv, (T *)a.o, a.lse, Bm, H, S, Dh);
        GemmArgs g = ga(M, d, d, a.o, d, nullptr, 0, a.x_mid, d);
        g.R = x_in;
        gemm_w(EPI_RESID, g, L.wo[l]);
        layernorm_fwd<T>(st, a.x_mid, params + L.g2[l], (T *)a.b, a.mean2, a.rstd2, M, d, c.ln_eps);
        g = ga(M, F, d, a.b, d, nullptr, 0, a.h, F);
        g.C2 = a.u;
        gemm_w(EPI_GELU, g, L.w1[l]);
        g = ga(M, d, F, a.u, F, nullptr, 0, x_out, d);
        g.R = a.x_mid;
        gemm_w(EPI_RESID, g, L.w2[l]);
    }

    // dx_in: gradient w.r.t. the block output (fp32) with its T copy in w.dx16; writes the
    // gradient w.r.t. the block input to dx_out (+ T copy in w.dx16).
    void block_backward(int l, const float *x_in, BlockActs &a, const float *dx_in, float *dx_out) {
        const Layout &L = w.lay;
        T *dx16 = (T *)w.dx16, *dff = (T *)w.dff, *dtmp = (T *)w.dtmp, *dqkv = (T *)w.dqkv;
        // MLP: x'' = x' + GELU(b W1) W2
        GemmArgs g = ga(F, d, M, a.u, F, dx16, d, grads + L.w2[l], d);
        g.beta = beta;
        gemm<T>(st, GEMM_TN, EPI_ACCUM, g);
        g = ga(M, F, d, dx16, d, wmat + L.w2[l], d, dff, F);
        g.H = a.h;
        gemm<T>(st, GEMM_NT, EPI_DGELU, g);
        g = ga(d, F, M, a.b, d, dff, F, grads + L.w1[l], F);
        g.beta = beta;
        gemm<T>(st, GEMM_TN, EPI_ACCUM, g);
        gemm<T>(st, GEMM_NT, EPI_STORE, ga(M, d, F, dff, F, wmat + L.w1[l], F, dtmp, d));
        layernorm_bwd<T>(st, dtmp, a.x_mid, a.mean2, a.rstd2, params + L.g2[l], dx_in, dx_out, dx16,
                         grads + L.g2[l], beta != 0.f, w.ln_scratch, M, d);
        // attention: x' = x + Attn(LN(x) Wqkv) Wo        (dx_out now holds dL/dx')
        gemm<T>(st, GEMM_NT, EPI_STORE, ga(M, d, d, dx16, d, wmat + L.wo[l], d, dtmp, d));
        attention_bwd<T>(st, (const T *)a.qkv, (const T *)a.o, a.lse, dtmp, dqkv, w.dvec, Bm, H, S, Dh);
        // dWqkv and dWo together: dx16 (dL/dx') stays intact until the LayerNorm backward below
        g = ga(d, 3 * d, M, a.a, d, dqkv, 3 * d, grads + L.wqkv[l], 3 * d);
        g.beta = beta;
        GemmArgs go = ga(d, d, M, a.o, d, dx16, d, grads + L.wo[l], d);
        go.beta = beta;
        gemm_tn_accum_pair<T>(st, g, go);
        gemm<T>(st, GEMM_NT, EPI_STORE, ga(M, d, 3 * d, dqkv, 3 * d, wmat + L.wqkv[l], 3 * d, dtmp, d));
        // in-place on dx_out is safe: each element is read (as dres) and written by the same thread
        layernorm_bwd<T>(st, dtmp, x_in, a.mean1, a.rstd1, params + L.g1[l], dx_out, dx_out, dx16,
                         grads + L.g1[l], beta != 0.f, w.ln_scratch, M, d);
    }

    // One micro-batch: adds its gradients (scaled by grad_scale / M) to beta * grads -- every
    // element of grads is written: the embedding by the head's weight-gradient product (before
    // the scatter-add of the input rows), every matrix by its weight-gradient product, every
    // gain by the LayerNorm backward -- and loss_scale * mean loss to *loss_acc.
    void micro_batch(const int32_t *tokens, float grad_scale, double loss_scale, double *loss_acc) {
        const Layout &L = w.lay;
        const int nl = c.n_layers;
        const bool recompute = c.recompute != 0;
        embedding_gather(st, params + L.E, tokens, w.x_in[0], Bm, S, d);
        for (int l = 0; l < nl; ++l) block_forward(l, w.x_in[l], w.acts[recompute ? 0 : l], w.x_in[l + 1]);

        // head: final LayerNorm, tied LM head, cross-entropy, chunked over rows
        T *y = (T *)w.y, *dy = (T *)w.dy, *z = (T *)w.logits;
        const T *E = wmat + L.E;
        layernorm_fwd<T>(st, w.x_in[nl], params + L.gf, y, w.meanf, w.rstdf, M, d, c.ln_eps);
        for (int m0 = 0; m0 < M; m0 += w.chunk) {
            const int rows = (M - m0) < w.chunk ? (M - m0) : w.chunk;
            gemm<T>(st, GEMM_NT, EPI_STORE, ga(rows, V, d, y + (int64_t)m0 * d, d, E, d, z, w.ldz));
            cross_entropy_fwd_bwd<T>(st, z, w.ldz, V, tokens, S, m0, rows, w.loss_rows, grad_scale / (float)M);
            gemm_w(EPI_STORE, ga(rows, d, V, z, w.ldz, nullptr, 0, dy + (int64_t)m0 * d, d), L.E);
            GemmArgs g = ga(V, d, rows, z, w.ldz, y + (int64_t)m0 * d, d, grads + L.E, d);
            g.beta = m0 == 0 ? beta : 1.f;  // later chunks of the same pass always accumulate
            gemm<T>(st, GEMM_TN, EPI_ACCUM, g);
        }
        loss_reduce(st, w.loss_rows, M, loss_scale / (double)M, loss_acc);
        layernorm_bwd<T>(st, dy, w.x_in[nl], w.meanf, w.rstdf, params + L.gf, nullptr, w.dx_a, (T *)w.dx16,
                         grads + L.gf, beta != 0.f, w.ln_scratch, M, d);

        float *dx_cur = w.dx_a, *dx_nxt = w.dx_b;
        for (int l = nl - 1; l >= 0; --l) {
            BlockActs &a = w.acts[recompute ? 0 : l];
            if (recompute) block_forward(l, w.x_in[l], a, w.x_in[l + 1]);  // re-run the block's forward
            block_backward(l, w.x_in[l], a, dx_cur, dx_nxt);
            float *t = dx_cur; dx_cur = dx_nxt; dx_nxt = t;
        }
        // per micro-batch of the ctx: the kernel's search for equal ids is quadratic in the rows
        // it is given, and this keeps the summation order that of unfused micro-batches
        const int mb = ctx->micro_batch;
        for (int b0 = 0; b0 < Bm; b0 += mb)
            embedding_scatter_add(st, dx_cur + (int64_t)b0 * S * d, tokens + (int64_t)b0 * (S + 1), grads + L.E,
                                  (Bm - b0) < mb ? (Bm - b0) : mb, S, d);
    }
};

template <typename T>
int alloc_workspace(photon_ctx *ctx) {
    ModelWorkspace &w = *ctx->ws;
    const photon_model_cfg &c = ctx->cfg;
    const int fuse = c.micro_fuse > 1 ? c.micro_fuse : 1;
    const int64_t M = (int64_t)ctx->micro_batch * fuse * c.seq_len, d = c.d_model, F = c.d_ff;
    const int nl = c.n_layers;
    const size_t ts = sizeof(T);
    w.tsize = ts;
    w.M = (int)M;
    // LM-head row chunk: at most 1 GiB of logits at a time.  Every chunk costs one read-modify-write
    // pass over the embedding gradient, so fewer and larger chunks are better; a 4 x 2048-token
    // micro-batch at vocabulary 50368 in bf16 (0.83 GB) is a single chunk.
    w.ldz = (c.vocab + 255) / 256 * 256;
    int64_t chunk = ((int64_t)1 << 30) / ((int64_t)w.ldz * (int64_t)ts);
    // whole multiples of 8192 rows where possible: the input-gradient product of a chunk
    // (rows x d_model, K = vocabulary) then has a multiple of 256 tiles at d_model = 2048, one
    // full wave of workgroups on the 256 compute units
    chunk = chunk >= 8192 ? chunk / 8192 * 8192 : chunk / 256 * 256;
    if (chunk < 256) chunk = 256;
    if (chunk > M) chunk = M;
    w.chunk = (int)chunk;

    if (ts == 2) {
        TRY_RC(dev_alloc(ctx, &w.w16, sizeof(bf16) * (size_t)(ctx->n + 64 * d)));
        TRY_RC(dev_alloc(ctx, &w.w16t, sizeof(bf16) * (size_t)(ctx->n + 64 * d)));
    }
    TRY_RC(dev_alloc(ctx, &w.grads, sizeof(float) * (size_t)ctx->n));
    w.x_in.resize(nl + 1);
    for (int l = 0; l <= nl; ++l) TRY_RC(dev_alloc(ctx, &w.x_in[l], sizeof(float) * (size_t)(M * d)));
    const int slots = c.recompute ? 1 : nl;
    w.acts.resize(slots);
    const int64_t BHS = (int64_t)ctx->micro_batch * fuse * c.n_heads * c.seq_len;
    for (int s = 0; s < slots; ++s) {
        BlockActs &a = w.acts[s];
        TRY_RC(dev_alloc(ctx, &a.a, ts * (size_t)(M * d)));
        TRY_RC(dev_alloc(ctx, &a.qkv, ts * (size_t)(M * 3 * d)));
        TRY_RC(dev_alloc(ctx, &a.o, ts * (size_t)(M * d)));
        TRY_RC(dev_alloc(ctx, &a.b, ts * (size_t)(M * d)));
        TRY_RC(dev_alloc(ctx, &a.h, ts * (size_t)(M * F)));
        TRY_RC(dev_alloc(ctx, &a.u, ts * (size_t)(M * F)));
        TRY_RC(dev_alloc(ctx, &a.x_mid, sizeof(float) * (size_t)(M * d)));
        TRY_RC(dev_alloc(ctx, &a.mean1, sizeof(float) * (size_t)M));
        TRY_RC(dev_alloc(ctx, &a.rstd1, sizeof(float) * (size_t)M));
        TRY_RC(dev_alloc(ctx, &a.mean2, sizeof(float) * (size_t)M));
        TRY_RC(dev_alloc(ctx, &a.rstd2, sizeof(float) * (size_t)M));
        TRY_RC(dev_alloc(ctx, &a.lse, sizeof(float) * (size_t)BHS));
    }
    TRY_RC(dev_alloc(ctx, &w.meanf, sizeof(float) * (size_t)M));
    TRY_RC(dev_alloc(ctx, &w.rstdf, sizeof(float) * (size_t)M));
    TRY_RC(dev_alloc(ctx, &w.y, ts * (size_t)(M * d)));
    TRY_RC(dev_alloc(ctx, &w.logits, ts * (size_t)((int64_t)w.chunk * w.ldz)));
    TRY_RC(dev_alloc(ctx, &w.loss_rows, sizeof(float) * (size_t)M));
    w.loss_cap = 4096;
    TRY_RC(dev_alloc(ctx, &w.loss_acc, sizeof(double) * (size_t)w.loss_cap));
    TRY_RC(dev_alloc(ctx, &w.tok_flag, 16));
    TRY_RC(dev_alloc(ctx, &w.dx_a, sizeof(float) * (size_t)(M * d)));
    TRY_RC(dev_alloc(ctx, &w.dx_b, sizeof(float) * (size_t)(M * d)));
    TRY_RC(dev_alloc(ctx, &w.dvec, sizeof(float) * (size_t)(2 * BHS)));
    TRY_RC(dev_alloc(ctx, &w.ln_scratch, sizeof(float) * (size_t)layernorm_bwd_scratch_floats((int)d)));
    TRY_RC(dev_alloc(ctx, &w.dx16, ts * (size_t)(M * d)));
    TRY_RC(dev_alloc(ctx, &w.dff, ts * (size_t)(M * F)));
    TRY_RC(dev_alloc(ctx, &w.dqkv, ts * (size_t)(M * 3 * d)));
    TRY_RC(dev_alloc(ctx, &w.dtmp, ts * (size_t)(M * d)));
    TRY_RC(dev_alloc(ctx, &w.dy, ts * (size_t)(M * d)));
    if (ts == 2) {
        // split-K partial tiles: up to 8 partials of the largest few-tile products (d x d, chunk x d)
        const int64_t big = d * d > (int64_t)w.chunk * d ? d * d : (int64_t)w.chunk * d;
        w.splitk_bytes = sizeof(float) * (size_t)(8 * big);
        TRY_RC(dev_alloc(ctx, &w.splitk, w.splitk_bytes));
        // every piece of the flat vector as a matrix: E [V, d], the weights, the gains as [1, d]
        const Layout &L = w.lay;
        std::vector<int64_t> off;
        std::vector<int> rows, cols;
        auto add = [&](int64_t o, int r, int cc) { off.push_back(o); rows.push_back(r); cols.push_back(cc); };
        add(L.E, c.vocab, (int)d);
        for (int l = 0; l < nl; ++l) {
            add(L.g1[l], 1, (int)d);
            add(L.wqkv[l], (int)d, (int)(3 * d));
            add(L.wo[l], (int)d, (int)d);
            add(L.g2[l], 1, (int)d);
            add(L.w1[l], (int)d, (int)F);
            add(L.w2[l], (int)F, (int)d);
        }
        add(L.gf, 1, (int)d);
        w.adam_mats = (int)off.size();
        TRY_RC(flat_adamw_table(ctx, off.data(), rows.data(), cols.data(), w.adam_mats, &w.adam_table, &w.adam_tiles));
        w.allocs.push_back(w.adam_table);
    }
    return PHOTON_OK;
}

// bf16 working copies of the weights after the masters changed: the flat copy is already in
// place (written by AdamW or by the conversion pass); this adds the transposed matrices.
void refresh_transposed(photon_ctx *ctx) {
    ModelWorkspace &w = *ctx->ws;
    const photon_model_cfg &c = ctx->cfg;
    const Layout &L = w.lay;
    hipStream_t st = ctx->stream;
    const int d = c.d_model, F = c.d_ff;
    transpose_bf16(st, w.w16 + L.E, w.w16t + L.E, c.vocab, d);
    for (int l = 0; l < c.n_layers; ++l) {
        transpose_bf16(st, w.w16 + L.wqkv[l], w.w16t + L.wqkv[l], d, 3 * d);
        transpose_bf16(st, w.w16 + L.wo[l], w.w16t + L.wo[l], d, d);
        transpose_bf16(st, w.w16 + L.w1[l], w.w16t + L.w1[l], d, F);
        transpose_bf16(st, w.w16 + L.w2[l], w.w16t + L.w2[l], F, d);
    }
}

// Token ids index rows of the embedding and of its gradient and columns of the logits: an id
// outside [0, vocab) would be an out-of-bounds access, so every id of a call is checked on the
// device before any model kernel runs (one pass over the ids, one 4-byte read-back).
int check_tokens(photon_ctx *ctx, const int32_t *tokens, int64_t count) {
    ModelWorkspace &w = *ctx->ws;
    hipStream_t st = ctx->stream;
    token_range_check(st, tokens, count, ctx->cfg.vocab, w.tok_flag);
    HIP_TRY(ctx, hipGetLastError());
    int bad = 0;
    HIP_TRY(ctx, hipMemcpyAsync(&bad, w.tok_flag, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    return bad ? PHOTON_EINVAL : PHOTON_OK;
}

template <typename T>
int run_loss_grad(photon_ctx *ctx, const float *params, const int32_t *tokens, float *grads, float *loss) {
    ModelWorkspace &w = *ctx->ws;
    hipStream_t st = ctx->stream;
    TRY_RC(check_tokens(ctx, tokens, (int64_t)ctx->micro_batch * (ctx->cfg.seq_len + 1)));
    if (sizeof(T) == 2) {
        convert_f32_to_bf16(st, params, w.w16, ctx->n);
        refresh_transposed(ctx);
    }
    fill_zero_f32(st, reinterpret_cast<float *>(w.loss_acc), 2);  // a fill kernel, not a memset node: safe under graph capture
    Runner<T> r(ctx, params, grads, ctx->micro_batch);
    r.beta = 0.f;  // grads_out is overwritten
    r.micro_batch(tokens, 1.0f, 1.0, w.loss_acc);
    HIP_TRY(ctx, hipGetLastError());
    double host = 0.0;
    HIP_TRY(ctx, hipMemcpyAsync(&host, w.loss_acc, sizeof(double), hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    *loss = (float)host;
    return std::isfinite(host) ? PHOTON_OK : PHOTON_ENONFINITE;
}

template <typename T>
int run_local_steps(photon_ctx *ctx, float *params, photon_opt_state *os, const int32_t *tokens, int n_steps,
                    int n_micro, const float *lrs, const photon_adamw_hp *hp, float *loss_out) {
    ModelWorkspace &w = *ctx->ws;
    hipStream_t st = ctx->stream;
    const photon_model_cfg &c = ctx->cfg;
    const int64_t mb_tokens = (int64_t)ctx->micro_batch * (c.seq_len + 1);
    // micro-batches fused per pass: the largest divisor of n_micro that the workspace holds
    int group = 1;
    for (int g = c.micro_fuse > 1 ? c.micro_fuse : 1; g > 1; --g)
        if (n_micro % g == 0) {
            group = g;
            break;
        }
    const int n_groups = n_micro / group;
    TRY_RC(check_tokens(ctx, tokens, (int64_t)n_steps * n_micro * mb_tokens));
    if (sizeof(T) == 2) {
        convert_f32_to_bf16(st, params, w.w16, ctx->n);
        refresh_transposed(ctx);
    }
    std::vector<double> host(n_steps);
    bool finite = true;
    for (int s0 = 0; s0 < n_steps; s0 += w.loss_cap) {
        const int ns = (n_steps - s0) < w.loss_cap ? (n_steps - s0) : w.loss_cap;
        fill_zero_f32(st, reinterpret_cast<float *>(w.loss_acc), 2 * (int64_t)ns);
        for (int s = 0; s < ns; ++s) {
            Runner<T> r(ctx, params, w.grads, ctx->micro_batch * group);
            for (int j = 0; j < n_groups; ++j) {
                r.beta = j == 0 ? 0.f : 1.f;  // the first pass of the step overwrites the accumulators
                r.micro_batch(tokens + ((int64_t)(s0 + s) * n_micro + (int64_t)j * group) * mb_tokens,
                              1.0f / (float)n_groups, 1.0 / (double)n_groups, w.loss_acc + s);
            }
            if (sizeof(T) == 2)  // one pass: parameters, moments, the bf16 copy and its transposes
                TRY_RC(flat_adamw_tiled(ctx, params, os->m, os->v, w.grads, ctx->n, os->step + 1, lrs[s0 + s], hp,
                                        w.w16, w.w16t, w.adam_table, w.adam_mats, w.adam_tiles));
            else
                TRY_RC(flat_adamw(ctx, params, os->m, os->v, w.grads, ctx->n, os->step + 1, lrs[s0 + s], hp, nullptr));
            os->step += 1;
        }
        HIP_TRY(ctx, hipGetLastError());
        HIP_TRY(ctx, hipMemcpyAsync(host.data() + s0, w.loss_acc, sizeof(double) * ns, hipMemcpyDeviceToHost, st));
        HIP_TRY(ctx, hipStreamSynchronize(st));
    }
    for (int s = 0; s < n_steps; ++s) {
        loss_out[s] = (float)host[s];
        finite = finite && std::isfinite(host[s]);
    }
    return finite ? PHOTON_OK : PHOTON_ENONFINITE;
}

}  // namespace

int model_create(photon_ctx *ctx) {
    const photon_model_cfg &c = ctx->cfg;
    if (c.d_model > 4096) return PHOTON_ENOTIMPL;  // LayerNorm kernels keep a row in registers
    ctx->ws = new (std::nothrow) ModelWorkspace();
    if (!ctx->ws) return PHOTON_ENOMEM;
    ctx->ws->lay = make_layout(c);
    if (ctx->ws->lay.total != ctx->n) return PHOTON_EINVAL;
    return c.compute_dtype == PHOTON_BF16 ? alloc_workspace<bf16>(ctx) : alloc_workspace<float>(ctx);
}

void model_destroy(photon_ctx *ctx) {
    if (!ctx->ws) return;
    for (void *p : ctx->ws->allocs) (void)hipFree(p);
    delete ctx->ws;
    ctx->ws = nullptr;
}

int model_local_steps(photon_ctx *ctx, float *params, photon_opt_state *st, const int32_t *tokens, int n_steps,
                      int n_micro, const float *lrs, const photon_adamw_hp *hp, float *loss_out) {
    return ctx->cfg.compute_dtype == PHOTON_BF16
               ? run_local_steps<bf16>(ctx, params, st, tokens, n_steps, n_micro, lrs, hp, loss_out)
               : run_local_steps<float>(ctx, params, st, tokens, n_steps, n_micro, lrs, hp, loss_out);
}

int model_loss_grad(photon_ctx *ctx, const float *params, const int32_t *tokens, float *grads, float *loss) {
    return ctx->cfg.compute_dtype == PHOTON_BF16 ? run_loss_grad<bf16>(ctx, params, tokens, grads, loss)
                                                 : run_loss_grad<float>(ctx, params, tokens, grads, loss);
}
