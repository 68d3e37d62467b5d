// Launchers of the model kernels.  T is the storage type of activations and matmul
// operands: float (everything in fp32) or bf16 (bf16 operands, fp32 accumulation); the
// residual stream, LayerNorm statistics, log-sum-exp values, the loss and every parameter
// gradient are fp32 in both modes.
#pragma once

#include "common.h"

// C[M,N] = op(A) op(B), row-major:
//   NN: A[M,K] B[K,N]      forward projections (weights stored [in, out])
//   NT: A[M,K] B[N,K]^T    input gradients dX = dY W^T, and the tied LM head y E^T
//   TN: A[K,M]^T B[K,N]    weight gradients dW = X^T dY
enum GemmOp { GEMM_NN = 0, GEMM_NT = 1, GEMM_TN = 2 };

enum GemmEpi {
    EPI_STORE = 0,  // C (T) = acc
    EPI_RESID = 1,  // C (fp32) = R (fp32) + acc            residual add of the block
    EPI_GELU = 2,   // h = acc: C (T) = GELU'(h), C2 (T) = GELU(h)   MLP up-projection; the derivative is
                    //                                       what the backward pass needs of h
    EPI_DGELU = 3,  // C (T) = acc * H, H = saved GELU'(h)   backward through the activation
    EPI_ACCUM = 4   // C (fp32) = beta * C + acc             weight-gradient accumulation
};

struct GemmArgs {
    int M = 0, N = 0, K = 0;
    const void *A = nullptr;
    int lda = 0;
    const void *B = nullptr;
    int ldb = 0;
    void *C = nullptr;
    int ldc = 0;
    const float *R = nullptr;  // EPI_RESID, leading dimension ldc
    void *C2 = nullptr;        // EPI_GELU, leading dimension ldc
    const void *H = nullptr;   // EPI_DGELU: saved GELU'(h), leading dimension ldc
    float beta = 0.f;          // EPI_ACCUM
};

template <typename T>
void gemm(hipStream_t st, GemmOp op, GemmEpi epi, const GemmArgs &g);
template <typename T>
void gemm_simple(hipStream_t st, GemmOp op, GemmEpi epi, const GemmArgs &g);
// bf16 MFMA path; returns false when the shape is not covered (caller falls back to gemm_simple).
bool gemm_mfma_bf16(hipStream_t st, GemmOp op, GemmEpi epi, const GemmArgs &g);
// Two TN / EPI_ACCUM products in one launch; false when the pair is not covered (the caller then
// issues them one by one).
bool gemm_mfma_bf16_pair_covered(const GemmArgs &g1, const GemmArgs &g2);
bool gemm_mfma_bf16_pair_tn_accum(hipStream_t st, const GemmArgs &g1, const GemmArgs &g2);
// dW1 += A1^T B1 and dW2 += A2^T B2 (both GEMM_TN, EPI_ACCUM), fused into one launch where it pays
template <typename T>
void gemm_tn_accum_pair(hipStream_t st, const GemmArgs &g1, const GemmArgs &g2);
// float32 scratch for split-K partial tiles (device memory, owned by the caller); none = no split-K.
// Per host thread: the caller sets it before the GEMMs of the ctx it runs.
void gemm_set_splitk_workspace(float *ws, size_t bytes);

// x0[m,:] = E[tok(m),:] for the M = B*S input positions; tokens are [B][S+1].
void embedding_gather(hipStream_t st, const float *E, const int32_t *tokens, float *x0, int B, int S, int d);
// dE[tok(m),:] += dx0[m,:], rows of one token summed in increasing m (deterministic).
void embedding_scatter_add(hipStream_t st, const float *dx0, const int32_t *tokens, float *dE, int B, int S, int d);

template <typename T>
void layernorm_fwd(hipStream_t st, const float *x, const float *gain, T *y, float *mean, float *rstd, int M, int d,
                   float eps);
// dx_out = (dres ? dres : 0) + LN'(dy); dx16 (optional) = T(dx_out);
// dgain = (accumulate ? dgain : 0) + column sums of dy * xhat.
template <typename T>
void layernorm_bwd(hipStream_t st, const T *dy, const float *x, const float *mean, const float *rstd,
                   const float *gain, const float *dres, float *dx_out, T *dx16, float *dgain, bool accumulate,
                   float *scratch, int M, int d);
int layernorm_bwd_scratch_floats(int d);

// Causal ALiBi attention on packed qkv [M, 3d] (q | k | v, head h at columns h*Dh).
// o: [M, d]; lse: [B, H, S].
template <typename T>
void attention_fwd(hipStream_t st, const T *qkv, T *o, float *lse, int B, int H, int S, int Dh);
// dqkv [M, 3d] from d_o [M, d]; dvec: scratch of 2 * B * H * S floats.
template <typename T>
void attention_bwd(hipStream_t st, const T *qkv, const T *o, const float *lse, const T *d_o, T *dqkv, float *dvec,
                   int B, int H, int S, int Dh);
template <typename T>
void attention_fwd_simple(hipStream_t st, const T *qkv, T *o, float *lse, int B, int H, int S, int Dh);
template <typename T>
void attention_bwd_simple(hipStream_t st, const T *qkv, const T *o, const float *lse, const T *d_o, T *dqkv,
                          float *dvec, int B, int H, int S, int Dh);
bool attention_fwd_flash_bf16(hipStream_t st, const bf16 *qkv, bf16 *o, float *lse, int B, int H, int S, int Dh);
bool attention_bwd_flash_bf16(hipStream_t st, const bf16 *qkv, const bf16 *o, const float *lse, const bf16 *d_o,
                              bf16 *dqkv, float *dvec, int B, int H, int S, int Dh);

// Softmax cross-entropy over rows [m0, m0 + rows) of the micro-batch: reads logits (row stride
// ldz, V valid columns), writes loss_rows[m] = lse - z_target and overwrites the logits with
// dz = (softmax - onehot) * scale (columns >= V up to ldz are set to 0).
template <typename T>
void cross_entropy_fwd_bwd(hipStream_t st, T *logits, int ldz, int V, const int32_t *tokens, int S, int m0, int rows,
                           float *loss_rows, float scale);
// acc[0] += scale * sum(loss_rows[0..M)) in a fixed order, float64.
void loss_reduce(hipStream_t st, const float *loss_rows, int M, double scale, double *acc);

// flag[0] (device) = 1 if any of the n ids lies outside [0, V), else 0.
void token_range_check(hipStream_t st, const int32_t *tokens, int64_t n, int V, int *flag);

void convert_f32_to_bf16(hipStream_t st, const float *src, bf16 *dst, int64_t n);
// dst [cols, rows] = transpose of src [rows, cols]
void transpose_bf16(hipStream_t st, const bf16 *src, bf16 *dst, int rows, int cols);
