/*
 * photon.h -- C ABI of the federated-round hot path on one MI355X (gfx950).
 *
 * Two operations, named after the paper's statement of the problem:
 *
 *   photon_client_local_steps   the TrainClient call of the execution pipeline
 *                               (Alg. 1, LLM Client procedure; Alg. 3, inner loop):
 *                               tau AdamW steps of a decoder-only transformer on the
 *                               client's token batches, starting from the broadcast model.
 *   photon_aggregate            the aggregator lines of Alg. 1 / step 3 of Alg. 3:
 *                               pseudo-gradients Delta_k = theta - theta_k, their weighted
 *                               mean, and the server optimizer (FedAvg / FedMom / Nesterov,
 *                               hyper-parameter appendix).
 *
 * Conventions
 *   - Every pointer is marked HOST or DEVICE.  Device buffers are owned by the caller
 *     (allocated with any HIP allocator, e.g. torch), 16-byte aligned, and must stay valid
 *     until the call returns.  The library owns only the workspace inside a photon_ctx,
 *     allocated once in photon_create* and freed in photon_destroy.
 *   - All kernels run on the HIP stream given at create time (NULL = the default stream).
 *     A call that writes HOST outputs synchronises that stream before it returns; the others
 *     only enqueue work.
 *   - Every function returning int returns a photon_status; nothing aborts, throws or prints.
 *   - A context is not thread-safe; distinct contexts are independent.
 *   - Flat parameter vector (float32, length photon_param_count):
 *       E[vocab, d] | per block: g1[d], Wqkv[d,3d], Wo[d,d], g2[d], W1[d,d_ff], W2[d_ff,d] | gf[d]
 *     matrices row-major [in, out]; Wqkv columns are [q | k | v], head h owns columns
 *     h*Dh .. (h+1)*Dh-1 of each third.  Gradients, AdamW moments, pseudo-gradients and the
 *     server momentum use the same layout.
 */
#ifndef PHOTON_H
#define PHOTON_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct photon_ctx photon_ctx; /* opaque */

typedef enum {
    PHOTON_OK = 0,
    PHOTON_EINVAL = -1,     /* null / misaligned pointer, bad size, bad configuration, bad weights */
    PHOTON_ENOMEM = -2,     /* workspace allocation failed */
    PHOTON_EHIP = -3,       /* a HIP call failed; raw code via photon_last_hip_error */
    PHOTON_ENONFINITE = -4, /* a step's loss was NaN or Inf (all steps were still run) */
    PHOTON_ENOTIMPL = -5,   /* combination not built */
    PHOTON_ELIMIT = -6      /* size beyond the fixed limit of photon_aggregate_static */
} photon_status;

typedef enum { PHOTON_FP32 = 0, PHOTON_BF16 = 1 } photon_dtype;

/* What photon_aggregate's client buffers hold. */
typedef enum {
    PHOTON_CLIENT_PARAMS = 0, /* theta_k, float32: Delta_k is formed on the fly */
    PHOTON_CLIENT_DELTAS = 1  /* Delta_k = theta - theta_k, float32 or bfloat16 */
} photon_client_kind;

/* Model of Table 4 (blocks, width, heads, expansion, vocabulary, sequence length):
 * pre-LayerNorm blocks (gain only), causal attention with ALiBi bias -2^(-8h/H) (i-j),
 * exact GELU, tied embedding / LM head, no bias vectors.  d_model % n_heads == 0. */
typedef struct {
    int32_t n_layers, d_model, n_heads, d_ff, vocab, seq_len;
    float ln_eps;          /* 1e-5 */
    int32_t compute_dtype; /* photon_dtype: FP32 = everything in float32;
                              BF16 = bf16 matmul operands with fp32 accumulation, fp32 master
                              weights, fp32 residual stream, statistics and loss */
    int32_t recompute;     /* 0 keep all activations; 1 keep only every block's input and re-run each
                              block's forward during backward (activation recomputation per block,
                              which is also what "full" recomputation means when the block is the
                              unit that is checkpointed); 2 is reserved for a coarser policy (inputs
                              of every r-th block only) and photon_create returns PHOTON_ENOTIMPL */
    int32_t micro_fuse;    /* 0 or 1: every micro-batch of a step is a pass of its own.  G > 1: the
                              workspace holds G micro-batches and photon_client_local_steps runs the
                              micro-batches of a step g at a time as one batch, g = the largest
                              divisor of n_micro not above G.  Loss and gradient are the same means
                              over the same tokens (float32 summation order differs); weights are
                              read and weight gradients accumulated once per pass instead of once
                              per micro-batch.  Sized for GPUs whose memory holds the activations
                              of a whole optimizer step. */
} photon_model_cfg;

/* AdamW of the local optimizer (betas (0.9, 0.95) in the paper's tables). */
typedef struct {
    float beta1, beta2, eps, weight_decay;
} photon_adamw_hp;

/* Optimizer state.  m, v: DEVICE float32[N], caller-owned, updated in place.
 * step = number of updates already applied (0 with zeroed m, v at the start of every round:
 * stateless local optimisation). Updated by the call. */
typedef struct {
    float *m, *v;
    int64_t step;
} photon_opt_state;

/* Server optimizer: b <- mu b + Delta; u = Delta + mu b (nesterov) or b; theta <- theta - eta_s u.
 * momentum: DEVICE float32[N], caller-owned, zero before the first round; may be NULL iff mu == 0.
 * round is incremented by photon_aggregate. */
typedef struct {
    float eta_s, mu;
    int32_t nesterov;
    float *momentum;
    int64_t round;
} photon_outer_opt;

#define PHOTON_MAX_CLIENTS 64

/* Squared L2 norms of the averaged pseudo-gradient and of each client's pseudo-gradient
 * Delta_k = theta - theta_k, taken against the model as it was before the server step
 * (AggMetrics).  Entries k >= K are zero. */
typedef struct {
    double delta_norm2;
    double client_norm2[PHOTON_MAX_CLIENTS];
} photon_agg_metrics;


/* Time and algorithmic work per kernel class, measured with HIP events around every launch of
 * the class on the ctx stream (photon_profile_begin .. photon_profile_end).  The ratios
 * flops / ms and bytes / ms are the "device FLOPs/s" (resp. bytes/s) that the paper's MFU
 * definition (errata appendix: MFU = device FLOPs/s / peak) divides by the hardware peak. */
typedef struct {
    double gemm_ms, gemm_flops;     /* bf16 MFMA GEMMs: 2 M N K per launch */
    double attn_ms, attn_flops;     /* attention forward + backward: causal triangle, 4 resp. 10 S^2 Dh / 2 per head */
    double adamw_ms, adamw_bytes;   /* fused AdamW: 28 B / parameter (+ 2 with the bf16 copy) */
    double agg_ms, agg_bytes;       /* aggregation: (client bytes) K + 8 (+ 8 with momentum) B / parameter */
    double delta_ms, delta_bytes;   /* pseudo-gradient export: 8 B read + 2 or 4 B written / parameter */
    int64_t gemm_launches, attn_launches, adamw_launches, agg_launches, delta_launches;  /* timed launches */
    int64_t gemm_launches_total, attn_launches_total;  /* all launches of the class, timed or not */
} photon_profile;

/* Length N of the flat parameter vector, or a negative photon_status for an invalid cfg. */
int64_t photon_param_count(const photon_model_cfg *cfg);

/* Creates a context for a model: allocates activations, gradient accumulators and (bf16 mode)
 * the bf16 working copy of the weights for micro-batches of `micro_batch` sequences.
 * hip_stream: a hipStream_t passed as void* (NULL = default stream).  *out receives the ctx. */
int photon_create(const photon_model_cfg *cfg, int32_t micro_batch, void *hip_stream, photon_ctx **out);

/* Creates a context for the flat-vector operations only (photon_adamw_step,
 * photon_export_delta, photon_aggregate) on vectors of n elements; no model workspace. */
int photon_create_flat(int64_t n, void *hip_stream, photon_ctx **out);

/* Frees the workspace.  NULL is allowed. */
void photon_destroy(photon_ctx *ctx);

/* Static description of a status code. */
const char *photon_strerror(int status);

/* Raw hipError_t of the last failing HIP call on this ctx (0 if none). */
int photon_last_hip_error(const photon_ctx *ctx);

/* Bytes of device workspace the ctx holds. */
int64_t photon_workspace_bytes(const photon_ctx *ctx);

/*
 * Part A -- TrainClient (Alg. 1; Alg. 3 inner loop): n_steps AdamW steps.
 *   params          DEVICE float32[N]; the client's model, updated in place (the caller copies
 *                   the broadcast model into it first).
 *   opt_state       HOST struct; m, v DEVICE float32[N].
 *   token_batches   DEVICE int32 [n_steps][n_micro][micro_batch][seq_len + 1], ids in [0, vocab);
 *                   inputs are [..., :seq_len], the target of position t is token t + 1.
 *                   An id outside the range returns PHOTON_EINVAL before any step runs (the
 *                   ids are checked on the device; this costs one stream synchronisation).
 *   n_micro         micro-batches whose gradients are averaged into one optimizer step.
 *   lr_schedule     HOST float[n_steps]: the learning rate of each step (the caller evaluates the
 *                   cosine / warm-up schedule over sequential steps).
 *   loss_out        HOST float[n_steps]: mean next-token cross-entropy over all tokens of each
 *                   step, evaluated before that step's update.
 * Returns PHOTON_ENONFINITE if any loss is not finite (all steps are still run).
 */
int photon_client_local_steps(photon_ctx *ctx, float *params, photon_opt_state *opt_state,
                              const int32_t *token_batches, int32_t n_steps, int32_t n_micro,
                              const float *lr_schedule, const photon_adamw_hp *hp, float *loss_out);

/*
 * Loss and gradient of ONE micro-batch, no update (the "compute loss / compute gradients" lines
 * of Alg. 3).  tokens: DEVICE int32 [micro_batch][seq_len + 1], ids in [0, vocab) (checked,
 * PHOTON_EINVAL otherwise).  grads_out: DEVICE float32[N], overwritten.  loss_out: HOST float[1].
 */
int photon_client_loss_grad(photon_ctx *ctx, const float *params, const int32_t *tokens,
                            float *grads_out, float *loss_out);

/*
 * One AdamW update of a flat vector from a given gradient (ClientOpt of Alg. 3):
 *   t = step + 1; m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2;
 *   p = p (1 - lr wd) - lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps).
 * params, grads: DEVICE float32[n]; bf16_out: DEVICE bfloat16[n] or NULL (rounded copy of the
 * updated params, round-to-nearest-even).  n must equal the ctx's vector length.
 */
int photon_adamw_step(photon_ctx *ctx, float *params, photon_opt_state *opt_state, const float *grads,
                      float lr, const photon_adamw_hp *hp, void *bf16_out);

/*
 * Pseudo-gradient of one client (Alg. 1): delta_out[i] = (dtype)(global[i] - client[i]),
 * subtraction in float32, bf16 by round-to-nearest-even.  All DEVICE, length N.
 */
int photon_export_delta(photon_ctx *ctx, const float *global_params, const float *client_params,
                        void *delta_out, int32_t dtype);

/*
 * Part B -- aggregation and server step (Alg. 1 aggregator lines; Alg. 3 step 3):
 *   Delta = sum_{k=0}^{K-1} (w_k / sum_j w_j) Delta_k   (float32 FMA chain in the order k = 0..K-1)
 *   theta <- ServerOpt(theta, Delta)                     (see photon_outer_opt)
 *   global_params   DEVICE float32[N], updated in place.
 *   client_bufs     HOST array of K DEVICE pointers; contents per `kind` / `dtype`
 *                   (PARAMS requires dtype FP32).  No client buffer may overlap global_params
 *                   or outer_opt->momentum, nor those two each other (PHOTON_EINVAL).
 *   client_weights  HOST double[K]: unnormalised, finite, >= 0, sum > 0 (equal weights give the
 *                   1/|C| mean of Alg. 1; token counts give the weighted FedAvg).
 *   outer_opt       HOST struct, see above; round is incremented.
 *   metrics         HOST, may be NULL; when given the call synchronises the stream.
 * 1 <= K <= PHOTON_MAX_CLIENTS.  The result is bit-identical between runs.
 */
int photon_aggregate(photon_ctx *ctx, float *global_params, const void *const *client_bufs, int32_t K,
                     int32_t kind, int32_t dtype, const double *client_weights,
                     photon_outer_opt *outer_opt, photon_agg_metrics *metrics);

/*
 * photon_aggregate for callers that cannot allocate device memory or synchronise: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same kernels and the
 * same results as photon_aggregate, bit for bit, but no context: the only scratch the aggregation
 * needs -- (K + 1) rows of 2048 float32 norm slots -- lives in a device array that is part of the
 * library image, (PHOTON_STATIC_MAX_CLIENTS + 1) x 2048 x 4 bytes = 136 KiB on every GPU the
 * library is used on, held until the process ends.  The call allocates nothing, frees nothing,
 * copies nothing to the host and does not synchronise; it only enqueues kernels on hip_stream
 * (a hipStream_t as void*, NULL = default stream) for the current device.
 *   n               length of the vectors (>= 1).
 *   global_params, client_bufs, kind, dtype, client_weights, outer_opt
 *                   as for photon_aggregate (same checks, same PHOTON_EINVAL cases).
 *   K               1 <= K <= PHOTON_STATIC_MAX_CLIENTS; a larger K (up to PHOTON_MAX_CLIENTS)
 *                   returns PHOTON_ELIMIT and does nothing.
 *   norms_out       DEVICE double[K + 1] or NULL: norms_out[0] = squared norm of the averaged
 *                   pseudo-gradient, norms_out[1 + k] = client k's (the photon_agg_metrics values),
 *                   written by the stream; the caller reads them after its own synchronisation.
 *   hip_error_out   HOST, may be NULL: raw hipError_t when PHOTON_EHIP is returned, else 0.
 * The first call on a device looks up the array's device address (hipGetSymbolAddress); make
 * that call outside stream capture.  All calls on one GPU share the array: calls that overlap in
 * time on the same GPU (different streams or threads) race on the norm slots -- theta and the
 * momentum are still right, the norms are not -- so serialise them.  The array keeps the last
 * call's contents; every slot a call reads is written by that call first, nothing needs clearing.
 */
#define PHOTON_STATIC_MAX_CLIENTS 16
int photon_aggregate_static(void *hip_stream, int64_t n, float *global_params, const void *const *client_bufs,
                            int32_t K, int32_t kind, int32_t dtype, const double *client_weights,
                            photon_outer_opt *outer_opt, double *norms_out, int32_t *hip_error_out);

/*
 * Global-norm clipping of one client update, the simplest member of the optional
 * post-processing pipeline applied to an update before it is sent (Sec. 3): scales delta
 * (DEVICE, float32 or bf16, length N) in place by min(1, max_norm / ||delta||).
 * norm_out: HOST double[1], the norm before clipping (may be NULL).
 */
int photon_clip_delta(photon_ctx *ctx, void *delta, int32_t dtype, double max_norm, double *norm_out);


/*
 * Client start of a round (Alg. 3: omega_{i,0} <- theta; stateless local optimisation of the
 * hyper-parameter appendix): client_params <- global_params, m <- 0, v <- 0, step <- 0.
 * All DEVICE float32[N]; enqueued on the ctx stream.
 */
int photon_client_init(photon_ctx *ctx, const float *global_params, float *client_params,
                       photon_opt_state *opt_state);

/* Starts (and resets) per-kernel-class timing on this ctx; see photon_profile. */
int photon_profile_begin(photon_ctx *ctx);
/* The same, timing only every `every`-th launch (in launch order, every >= 1) of the GEMM and of
 * the attention class: an event pair costs a few microseconds of stream time, and these classes
 * have thousands of launches per optimizer step.  ms, flops and launches then cover the timed
 * launches only, so flops / ms remains the class's average rate; *_launches_total counts all. */
int photon_profile_begin_sampled(photon_ctx *ctx, int32_t every);
/* Synchronises the stream, fills *out (HOST) and stops timing. */
int photon_profile_end(photon_ctx *ctx, photon_profile *out);

/*
 * Measurement aid: what the memory system gives a plain streaming kernel shaped like the
 * flat-vector kernels of this library (16 bytes per lane and access, 2048 workgroups in grid
 * strides).  Every thread reads `reads` float32 vectors of length n (src, src + n, ...), adds them
 * and writes the sum to `writes` vectors (dst, dst + n, ...); reads, writes in 0..4, not both 0.
 * The mixes of the library's own kernels are 4 : 3.5 (AdamW), 2 : 0.5 (pseudo-gradient export),
 * 1 : 3 (client start) and (K / 2 + 1) : 1 (aggregation of K bf16 pseudo-gradients).
 *   src     DEVICE float32[reads * n] (may be NULL when reads == 0); dst DEVICE float32[max(writes, 1) * n]
 *   n       multiple of 4;  repeats >= 1 timed launches after one untimed
 *   ms_out  HOST double[1]: average milliseconds per launch; bytes moved = 4 n (reads + writes)
 * Synchronises the ctx stream.
 */
int photon_stream_probe(photon_ctx *ctx, int32_t reads, int32_t writes, const float *src, float *dst, int64_t n,
                        int32_t repeats, double *ms_out);

#ifdef __cplusplus
}
#endif
#endif /* PHOTON_H */
