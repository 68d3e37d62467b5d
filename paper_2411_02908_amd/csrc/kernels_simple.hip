// Shape-generic kernels of the transformer forward / backward pass: LayerNorm, embedding
// gather and deterministic scatter-add, softmax cross-entropy, and the plain (non-MFMA)
// GEMM and attention used for the fp32 mode and for shapes the MFMA kernels do not cover.
// The model is the pre-LayerNorm, ALiBi, GELU, tied-embedding decoder of Table 4.

#include "kernels.h"

namespace {

constexpr float kInvSqrt2 = 0.70710678118654752440f;
constexpr float kInvSqrt2Pi = 0.39894228040143267794f;

__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.0f + erff(x * kInvSqrt2)); }
__device__ __forceinline__ float gelu_grad_f(float x) {
    return 0.5f * (1.0f + erff(x * kInvSqrt2)) + x * __expf(-0.5f * x * x) * kInvSqrt2Pi;
}

// ------------------------------------------------------------------------------------ GEMM (plain)

constexpr int GT = 64;   // tile edge
constexpr int GK = 16;   // k step

template <typename T, int OP>
__global__ __launch_bounds__(256) void gemm_simple_kernel(GemmArgs g, int epi) {
    __shared__ float As[GK][GT + 4];
    __shared__ float Bs[GK][GT + 4];
    const T *A = reinterpret_cast<const T *>(g.A);
    const T *B = reinterpret_cast<const T *>(g.B);
    const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < g.K; k0 += GK) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int e = threadIdx.x + 256 * r;
            int m, k;
            float va = 0.f;
            if (OP == GEMM_TN) { k = e / GT; m = e % GT; } else { m = e / GK; k = e % GK; }
            if (m0 + m < g.M && k0 + k < g.K)
                va = to_f32(OP == GEMM_TN ? A[(int64_t)(k0 + k) * g.lda + m0 + m] : A[(int64_t)(m0 + m) * g.lda + k0 + k]);
            As[k][m] = va;
            int n;
            float vb = 0.f;
            if (OP == GEMM_NT) { n = e / GK; k = e % GK; } else { k = e / GT; n = e % GT; }
            if (n0 + n < g.N && k0 + k < g.K)
                vb = to_f32(OP == GEMM_NT ? B[(int64_t)(n0 + n) * g.ldb + k0 + k] : B[(int64_t)(k0 + k) * g.ldb + n0 + n]);
            Bs[k][n] = vb;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = m0 + ty * 4 + i;
        if (row >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + tx * 4 + j;
            if (col >= g.N) continue;
            const int64_t idx = (int64_t)row * g.ldc + col;
            const float v = acc[i][j];
            switch (epi) {
                case EPI_STORE: reinterpret_cast<T *>(g.C)[idx] = from_f32<T>(v); break;
                case EPI_RESID: reinterpret_cast<float *>(g.C)[idx] = g.R[idx] + v; break;
                case EPI_GELU:
                    reinterpret_cast<T *>(g.C)[idx] = from_f32<T>(gelu_grad_f(v));
                    reinterpret_cast<T *>(g.C2)[idx] = from_f32<T>(gelu_f(v));
                    break;
                case EPI_DGELU:
                    reinterpret_cast<T *>(g.C)[idx] = from_f32<T>(v * to_f32(reinterpret_cast<const T *>(g.H)[idx]));
                    break;
                default: {
                    float *c = reinterpret_cast<float *>(g.C) + idx;
                    *c = (g.beta != 0.f ? g.beta * *c : 0.f) + v;
                } break;
            }
        }
    }
}

// ------------------------------------------------------------------------------------ embedding

__global__ __launch_bounds__(256) void embedding_gather_kernel(const float *__restrict__ E,
                                                                const int32_t *__restrict__ tokens,
                                                                float *__restrict__ x0, int S, int d) {
    const int m = blockIdx.x;
    const int tok = tokens[(m / S) * (S + 1) + (m % S)];
    const f32x4 *src = reinterpret_cast<const f32x4 *>(E + (int64_t)tok * d);
    f32x4 *dst = reinterpret_cast<f32x4 *>(x0 + (int64_t)m * d);
    for (int c = threadIdx.x; c < d / 4; c += 256) dst[c] = src[c];
}

// One workgroup per input position m and slice of 1024 columns.  The first position holding a
// token id owns that id's row of dE: it collects the later positions with the same id, in
// increasing order, into an LDS list (ordered compaction, 256 positions at a time) and then adds
// their rows in that order -- a fixed summation order without atomics.  The frequent ids of a
// Zipf stream make chains of hundreds of rows that one workgroup walks alone: sixteen row loads
// are in flight per thread and the columns are split over workgroups, so that such a chain is
// bound by bandwidth, not by one memory latency per row.
constexpr int SCATTER_LIST = 4096;
constexpr int SCATTER_COLS = 1024;
__global__ __launch_bounds__(256) void embedding_scatter_kernel(const float *__restrict__ dx0,
                                                                 const int32_t *__restrict__ tokens,
                                                                 float *__restrict__ dE, int S, int M, int d) {
    __shared__ int earlier;
    __shared__ int list[SCATTER_LIST];
    __shared__ int wave_cnt[4];
    const int m = blockIdx.x;
    const int mb = m / S, ms = m - mb * S;
    const int tok = tokens[mb * (S + 1) + ms];
    if (threadIdx.x == 0) earlier = 0;
    __syncthreads();
    // does an earlier position hold the same id?  (rows of S + 1 ids, the last one a target only)
    int found = 0;
    for (int b = 0; b <= mb; ++b) {
        const int32_t *row = tokens + b * (S + 1);
        const int n = b < mb ? S : ms;
        for (int p = threadIdx.x; p < n; p += 256) found |= (row[p] == tok);
    }
    if (found) earlier = 1;
    __syncthreads();
    if (earlier) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.y * SCATTER_COLS + 4 * threadIdx.x;  // this thread's four columns
    const bool live = c < d;
    f32x4 acc = live ? *reinterpret_cast<const f32x4 *>(dE + (int64_t)tok * d + c) : f32x4{0.f, 0.f, 0.f, 0.f};
    int p0 = m;
    while (p0 < M) {
        // fill the list with matching positions from p0 on, in order
        int base = 0;
        while (p0 < M && base + 256 <= SCATTER_LIST) {
            const int p = p0 + threadIdx.x;
            const int pb = p / S;
            const bool hit = p < M && tokens[pb * (S + 1) + (p - pb * S)] == tok;
            const unsigned long long mask = __ballot(hit);
            const int before = __popcll(mask & ((1ull << lane) - 1ull));
            if (lane == 0) wave_cnt[wave] = __popcll(mask);
            __syncthreads();
            int off = base;
            for (int w = 0; w < wave; ++w) off += wave_cnt[w];
            if (hit) list[off + before] = p;
            base += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
            __syncthreads();
            p0 += 256;
        }
        // rows are added in list order, sixteen loads in flight
        constexpr int UR = 16;
        for (int q0 = 0; q0 < base; q0 += UR) {
            f32x4 r[UR];
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                const int q = q0 + u < base ? q0 + u : base - 1;
                if (live) r[u] = *reinterpret_cast<const f32x4 *>(dx0 + (int64_t)list[q] * d + c);
            }
#pragma unroll
            for (int u = 0; u < UR; ++u)
                if (live && q0 + u < base) acc += r[u];
        }
        __syncthreads();
    }
    if (live) *reinterpret_cast<f32x4 *>(dE + (int64_t)tok * d + c) = acc;
}

// ------------------------------------------------------------------------------------ LayerNorm

constexpr int LN_THREADS = 256;
constexpr int LN_MAXC = 16;  // columns per thread: d <= 4096

template <typename T>
__global__ __launch_bounds__(LN_THREADS) void layernorm_fwd_kernel(const float *__restrict__ x,
                                                                    const float *__restrict__ gain, T *__restrict__ y,
                                                                    float *__restrict__ mean, float *__restrict__ rstd,
                                                                    int d, float eps) {
    __shared__ float red[LN_THREADS / PHOTON_WAVE];
    const int m = blockIdx.x;
    const float *xr = x + (int64_t)m * d;
    float v[LN_MAXC];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
        const int c = threadIdx.x + i * LN_THREADS;
        v[i] = c < d ? xr[c] : 0.f;
        s += v[i];
    }
    const float mu = block_sum<LN_THREADS>(s, red) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
        const int c = threadIdx.x + i * LN_THREADS;
        const float t = c < d ? v[i] - mu : 0.f;
        q += t * t;
    }
    const float rs = rsqrtf(block_sum<LN_THREADS>(q, red) / (float)d + eps);
    if (threadIdx.x == 0) {
        mean[m] = mu;
        rstd[m] = rs;
    }
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
        const int c = threadIdx.x + i * LN_THREADS;
        if (c < d) y[(int64_t)m * d + c] = from_f32<T>((v[i] - mu) * rs * gain[c]);
    }
}

// One wavefront per row (d = 256 NI): the row lives in registers as NI float4 per lane, both
// statistics are wave-level reductions (no workgroup barrier), all global traffic is 16 bytes per
// lane.  Same arithmetic as layernorm_fwd_kernel: mean, then the variance of the centred values.
template <typename T, int NI>
__global__ __launch_bounds__(256) void layernorm_fwd_wave_kernel(const float *__restrict__ x,
                                                                  const float *__restrict__ gain, T *__restrict__ y,
                                                                  float *__restrict__ mean, float *__restrict__ rstd,
                                                                  int M, float eps) {
    constexpr int D = NI * 256;
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    const float *xr = x + (int64_t)m * D;
    f32x4 v[NI];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        v[i] = *reinterpret_cast<const f32x4 *>(xr + 4 * (lane + 64 * i));
        s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
    }
    const float mu = wave_sum(s) * (1.0f / (float)D);
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[i][k] -= mu;
            q = fmaf(v[i][k], v[i][k], q);
        }
    const float rs = rsqrtf(wave_sum(q) * (1.0f / (float)D) + eps);
    if (lane == 0) {
        mean[m] = mu;
        rstd[m] = rs;
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int c = 4 * (lane + 64 * i);
        const f32x4 gn = *reinterpret_cast<const f32x4 *>(gain + c);
        if constexpr (sizeof(T) == 2) {
            bf16x4 o;
#pragma unroll
            for (int k = 0; k < 4; ++k) o[k] = (bf16)(v[i][k] * rs * gn[k]);
            *reinterpret_cast<bf16x4 *>(y + (int64_t)m * D + c) = o;
        } else {
            f32x4 o;
#pragma unroll
            for (int k = 0; k < 4; ++k) o[k] = v[i][k] * rs * gn[k];
            *reinterpret_cast<f32x4 *>(y + (int64_t)m * D + c) = o;
        }
    }
}

// Workgroup r walks rows r, r + G, ...; thread t owns columns t, t + 256, ... and keeps their
// gain-gradient sums in registers; partial[r][c] is combined over r in order by colsum_kernel.
template <typename T>
__global__ __launch_bounds__(LN_THREADS) void layernorm_bwd_kernel(
    const T *__restrict__ dy, const float *__restrict__ x, const float *__restrict__ mean,
    const float *__restrict__ rstd, const float *__restrict__ gain, const float *dres,
    float *dx_out, T *__restrict__ dx16, float *__restrict__ partial, int M, int d) {
    __shared__ float red[LN_THREADS / PHOTON_WAVE];
    float gn[LN_MAXC], dg[LN_MAXC];
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
        const int c = threadIdx.x + i * LN_THREADS;
        gn[i] = c < d ? gain[c] : 0.f;
        dg[i] = 0.f;
    }
    for (int m = blockIdx.x; m < M; m += gridDim.x) {
        const float mu = mean[m], rs = rstd[m];
        float xh[LN_MAXC], dxh[LN_MAXC];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < LN_MAXC; ++i) {
            const int c = threadIdx.x + i * LN_THREADS;
            if (c < d) {
                const float g = to_f32(dy[(int64_t)m * d + c]);
                xh[i] = (x[(int64_t)m * d + c] - mu) * rs;
                dxh[i] = g * gn[i];
                dg[i] += g * xh[i];
                s1 += dxh[i];
                s2 += dxh[i] * xh[i];
            } else {
                xh[i] = 0.f;
                dxh[i] = 0.f;
            }
        }
        const float m1 = block_sum<LN_THREADS>(s1, red) / (float)d;
        const float m2 = block_sum<LN_THREADS>(s2, red) / (float)d;
#pragma unroll
        for (int i = 0; i < LN_MAXC; ++i) {
            const int c = threadIdx.x + i * LN_THREADS;
            if (c < d) {
                float r = rs * (dxh[i] - m1 - xh[i] * m2);
                if (dres) r += dres[(int64_t)m * d + c];
                dx_out[(int64_t)m * d + c] = r;
                if (dx16) dx16[(int64_t)m * d + c] = from_f32<T>(r);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
        const int c = threadIdx.x + i * LN_THREADS;
        if (c < d) partial[(int64_t)blockIdx.x * d + c] = dg[i];
    }
}

// One wavefront per row (d = 256 NI <= 2560): the row lives in registers as NI float4 per lane,
// row statistics need only wave-level reductions (no workgroup barrier per row), and all global
// traffic is 16-byte per lane.  Wave w of the grid walks rows w, w + W, ...; the four waves of a
// workgroup combine their gain-gradient sums through LDS into partial[block][c].
template <typename T, int NI>
__global__ __launch_bounds__(256) void layernorm_bwd_wave_kernel(
    const T *__restrict__ dy, const float *__restrict__ x, const float *__restrict__ mean,
    const float *__restrict__ rstd, const float *__restrict__ gain, const float *dres, float *dx_out,
    T *__restrict__ dx16, float *__restrict__ partial, int M) {
    constexpr int D = NI * 256;
    __shared__ float red[3][D];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int gw = blockIdx.x * 4 + wave, nw = gridDim.x * 4;
    f32x4 gn[NI], dg[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        gn[i] = *reinterpret_cast<const f32x4 *>(gain + 4 * (lane + 64 * i));
        dg[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int m = gw; m < M; m += nw) {
        const float mu = mean[m], rs = rstd[m];
        const float *xr = x + (int64_t)m * D;
        const T *gr = dy + (int64_t)m * D;
        f32x4 xh[NI], dxh[NI];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int c = 4 * (lane + 64 * i);
            const f32x4 xv = *reinterpret_cast<const f32x4 *>(xr + c);
            f32x4 g;
            if constexpr (sizeof(T) == 2) {
                const bf16x4 gb = *reinterpret_cast<const bf16x4 *>(gr + c);
#pragma unroll
                for (int k = 0; k < 4; ++k) g[k] = (float)gb[k];
            } else {
                g = *reinterpret_cast<const f32x4 *>(gr + c);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                xh[i][k] = (xv[k] - mu) * rs;
                dxh[i][k] = g[k] * gn[i][k];
                dg[i][k] = fmaf(g[k], xh[i][k], dg[i][k]);
                s1 += dxh[i][k];
                s2 = fmaf(dxh[i][k], xh[i][k], s2);
            }
        }
        const float m1 = wave_sum(s1) * (1.0f / (float)D);
        const float m2 = wave_sum(s2) * (1.0f / (float)D);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int c = 4 * (lane + 64 * i);
            f32x4 r;
#pragma unroll
            for (int k = 0; k < 4; ++k) r[k] = rs * (dxh[i][k] - m1 - xh[i][k] * m2);
            if (dres) r += *reinterpret_cast<const f32x4 *>(dres + (int64_t)m * D + c);
            *reinterpret_cast<f32x4 *>(dx_out + (int64_t)m * D + c) = r;
            if (dx16) {
                if constexpr (sizeof(T) == 2) {
                    bf16x4 o;
#pragma unroll
                    for (int k = 0; k < 4; ++k) o[k] = (bf16)r[k];
                    *reinterpret_cast<bf16x4 *>(dx16 + (int64_t)m * D + c) = o;
                } else {
                    *reinterpret_cast<f32x4 *>(dx16 + (int64_t)m * D + c) = r;
                }
            }
        }
    }
    // waves 1..3 park their sums in LDS, wave 0 adds them in order and writes the block's row
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) *reinterpret_cast<f32x4 *>(&red[wave - 1][4 * (lane + 64 * i)]) = dg[i];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int c = 4 * (lane + 64 * i);
            f32x4 t = dg[i];
            t += *reinterpret_cast<const f32x4 *>(&red[0][c]);
            t += *reinterpret_cast<const f32x4 *>(&red[1][c]);
            t += *reinterpret_cast<const f32x4 *>(&red[2][c]);
            *reinterpret_cast<f32x4 *>(partial + (int64_t)blockIdx.x * D + c) = t;
        }
    }
}

// out[c] = (accumulate ? out[c] : 0) + sum_r partial[r][c].  16 columns per workgroup (64-byte row pieces), 16 interleaved
// row classes per column summed in increasing row order, classes then combined by a fixed tree:
// a fixed summation order with d / 16 workgroups in flight.
__global__ __launch_bounds__(256) void colsum_accum_kernel(const float *__restrict__ partial, int rows, int d,
                                                            float *__restrict__ out, bool accumulate) {
    __shared__ float red[16][17];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int c = blockIdx.x * 16 + tx;
    float s = 0.f;
    if (c < d)
        for (int r = ty; r < rows; r += 16) s += partial[(int64_t)r * d + c];
    red[ty][tx] = s;
    __syncthreads();
    for (int w = 8; w > 0; w >>= 1) {
        if (ty < w) red[ty][tx] += red[ty + w][tx];
        __syncthreads();
    }
    if (ty == 0 && c < d) out[c] = (accumulate ? out[c] : 0.f) + red[0][tx];
}

// ------------------------------------------------------------------------------------ attention (plain)

template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_simple_kernel(const T *__restrict__ qkv, T *__restrict__ o,
                                                              float *__restrict__ lse, int H, int S, int Dh) {
    extern __shared__ float sm[];
    float *sc = sm;        // [S]
    float *qs = sm + S;    // [Dh]
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int d = H * Dh, ld = 3 * d;
    const T *base = qkv + (int64_t)b * S * ld;
    const float scale = rsqrtf((float)Dh);
    const float slope = exp2f(-8.0f * (float)(h + 1) / (float)H);
    for (int c = lane; c < Dh; c += 64) qs[c] = to_f32(base[(int64_t)i * ld + h * Dh + c]);
    __syncthreads();
    float mx = -INFINITY;
    for (int j = lane; j <= i; j += 64) {
        const T *kr = base + (int64_t)j * ld + d + h * Dh;
        float s = 0.f;
        for (int c = 0; c < Dh; ++c) s = fmaf(qs[c], to_f32(kr[c]), s);
        s = s * scale - slope * (float)(i - j);
        sc[j] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = lane; j <= i; j += 64) {
        const float p = __expf(sc[j] - mx);
        sc[j] = p;
        sum += p;
    }
    sum = wave_sum(sum);
    __syncthreads();
    if (lane == 0) lse[((int64_t)b * H + h) * S + i] = mx + __logf(sum);
    const float inv = 1.0f / sum;
    for (int c = lane; c < Dh; c += 64) {
        float acc = 0.f;
        for (int j = 0; j <= i; ++j) acc = fmaf(sc[j], to_f32(base[(int64_t)j * ld + 2 * d + h * Dh + c]), acc);
        o[((int64_t)b * S + i) * d + h * Dh + c] = from_f32<T>(acc * inv);
    }
}

// dq_i and D_i = do_i . o_i
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dq_simple_kernel(const T *__restrict__ qkv, const T *__restrict__ o,
                                                                 const float *__restrict__ lse,
                                                                 const T *__restrict__ d_o, T *__restrict__ dqkv,
                                                                 float *__restrict__ dvec, int H, int S, int Dh) {
    extern __shared__ float sm[];
    float *sc = sm;             // [S] ds_ij
    float *qs = sm + S;         // [Dh]
    float *dos = sm + S + Dh;   // [Dh]
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int d = H * Dh, ld = 3 * d;
    const T *base = qkv + (int64_t)b * S * ld;
    const float scale = rsqrtf((float)Dh);
    const float slope = exp2f(-8.0f * (float)(h + 1) / (float)H);
    float dd = 0.f;
    for (int c = lane; c < Dh; c += 64) {
        qs[c] = to_f32(base[(int64_t)i * ld + h * Dh + c]);
        const float g = to_f32(d_o[((int64_t)b * S + i) * d + h * Dh + c]);
        dos[c] = g;
        dd = fmaf(g, to_f32(o[((int64_t)b * S + i) * d + h * Dh + c]), dd);
    }
    dd = wave_sum(dd);
    if (lane == 0) dvec[((int64_t)b * H + h) * S + i] = dd;
    __syncthreads();
    const float l = lse[((int64_t)b * H + h) * S + i];
    for (int j = lane; j <= i; j += 64) {
        const T *kr = base + (int64_t)j * ld + d + h * Dh;
        const T *vr = base + (int64_t)j * ld + 2 * d + h * Dh;
        float s = 0.f, dp = 0.f;
        for (int c = 0; c < Dh; ++c) {
            s = fmaf(qs[c], to_f32(kr[c]), s);
            dp = fmaf(dos[c], to_f32(vr[c]), dp);
        }
        const float p = __expf(s * scale - slope * (float)(i - j) - l);
        sc[j] = p * (dp - dd);
    }
    __syncthreads();
    for (int c = lane; c < Dh; c += 64) {
        float acc = 0.f;
        for (int j = 0; j <= i; ++j) acc = fmaf(sc[j], to_f32(base[(int64_t)j * ld + d + h * Dh + c]), acc);
        dqkv[((int64_t)b * S + i) * ld + h * Dh + c] = from_f32<T>(acc * scale);
    }
}

// dk_j, dv_j
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dkv_simple_kernel(const T *__restrict__ qkv,
                                                                  const float *__restrict__ lse,
                                                                  const T *__restrict__ d_o, T *__restrict__ dqkv,
                                                                  const float *__restrict__ dvec, int H, int S,
                                                                  int Dh) {
    extern __shared__ float sm[];
    float *sp = sm;                 // [S] p_ij
    float *sds = sm + S;            // [S] ds_ij
    float *ks = sm + 2 * S;         // [Dh]
    float *vs = sm + 2 * S + Dh;    // [Dh]
    const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int d = H * Dh, ld = 3 * d;
    const T *base = qkv + (int64_t)b * S * ld;
    const float scale = rsqrtf((float)Dh);
    const float slope = exp2f(-8.0f * (float)(h + 1) / (float)H);
    for (int c = lane; c < Dh; c += 64) {
        ks[c] = to_f32(base[(int64_t)j * ld + d + h * Dh + c]);
        vs[c] = to_f32(base[(int64_t)j * ld + 2 * d + h * Dh + c]);
    }
    __syncthreads();
    for (int i = j + lane; i < S; i += 64) {
        const T *qr = base + (int64_t)i * ld + h * Dh;
        const T *gr = d_o + ((int64_t)b * S + i) * d + h * Dh;
        float s = 0.f, dp = 0.f;
        for (int c = 0; c < Dh; ++c) {
            s = fmaf(to_f32(qr[c]), ks[c], s);
            dp = fmaf(to_f32(gr[c]), vs[c], dp);
        }
        const int64_t li = ((int64_t)b * H + h) * S + i;
        const float p = __expf(s * scale - slope * (float)(i - j) - lse[li]);
        sp[i - j] = p;
        sds[i - j] = p * (dp - dvec[li]);
    }
    __syncthreads();
    for (int c = lane; c < Dh; c += 64) {
        float dk = 0.f, dv = 0.f;
        for (int i = j; i < S; ++i) {
            dk = fmaf(sds[i - j], to_f32(base[(int64_t)i * ld + h * Dh + c]), dk);
            dv = fmaf(sp[i - j], to_f32(d_o[((int64_t)b * S + i) * d + h * Dh + c]), dv);
        }
        dqkv[((int64_t)b * S + j) * ld + d + h * Dh + c] = from_f32<T>(dk * scale);
        dqkv[((int64_t)b * S + j) * ld + 2 * d + h * Dh + c] = from_f32<T>(dv);
    }
}

// ------------------------------------------------------------------------------------ cross-entropy

// One workgroup per row.  Pass 1 keeps a running (max, sum of exp) per thread over 8-element
// vectors and merges them across the workgroup; pass 2 rewrites the row (still hot in L2) as
// (softmax - onehot) * scale.  The full-vocabulary probabilities never exist anywhere else.
template <typename T>
__global__ __launch_bounds__(256) void cross_entropy_kernel(T *__restrict__ logits, int ldz, int V,
                                                             const int32_t *__restrict__ tokens, int S, int m0,
                                                             float *__restrict__ loss_rows, float scale) {
    __shared__ float red[256 / PHOTON_WAVE];
    constexpr int VEC = 16 / sizeof(T);
    typedef T vec_t __attribute__((ext_vector_type(VEC)));
    const int m = m0 + blockIdx.x;
    T *z = logits + (int64_t)blockIdx.x * ldz;
    const int tgt = tokens[(m / S) * (S + 1) + (m % S) + 1];
    const int nvec = V / VEC;
    float mx = -INFINITY, sum = 0.f;
    for (int i = threadIdx.x; i < nvec; i += 256) {
        const vec_t v = *reinterpret_cast<const vec_t *>(z + i * VEC);
        float lm = to_f32(v[0]);
#pragma unroll
        for (int k = 1; k < VEC; ++k) lm = fmaxf(lm, to_f32(v[k]));
        if (lm > mx) {
            sum *= __expf(mx - lm);
            mx = lm;
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) sum += __expf(to_f32(v[k]) - mx);
    }
    for (int c = nvec * VEC + threadIdx.x; c < V; c += 256) {
        const float x = to_f32(z[c]);
        if (x > mx) {
            sum *= __expf(mx - x);
            mx = x;
        }
        sum += __expf(x - mx);
    }
    const float gmx = block_max<256>(mx, red);
    const float gsum = block_sum<256>(mx == -INFINITY ? 0.f : sum * __expf(mx - gmx), red);
    const float lse = gmx + __logf(gsum);
    if (threadIdx.x == 0) loss_rows[m] = lse - to_f32(z[tgt]);
    __syncthreads();
    for (int i = threadIdx.x; i < nvec; i += 256) {
        vec_t v = *reinterpret_cast<const vec_t *>(z + i * VEC);
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const int c = i * VEC + k;
            v[k] = from_f32<T>((__expf(to_f32(v[k]) - lse) - (c == tgt ? 1.0f : 0.0f)) * scale);
        }
        *reinterpret_cast<vec_t *>(z + i * VEC) = v;
    }
    for (int c = nvec * VEC + threadIdx.x; c < ldz; c += 256) {
        float g = 0.f;
        if (c < V) g = (__expf(to_f32(z[c]) - lse) - (c == tgt ? 1.0f : 0.0f)) * scale;
        z[c] = from_f32<T>(g);
    }
}

// The same with the row held in registers between the two passes (NV 16-byte vectors per thread,
// V <= 256 * NV * VEC): the second pass of the kernel above finds its row neither in L2 nor, with
// thousands of 100 KB rows in flight, reliably in the last-level cache, so it costs a third read.
template <typename T, int NV>
__global__ __launch_bounds__(256) void cross_entropy_regs_kernel(T *__restrict__ logits, int ldz, int V,
                                                                  const int32_t *__restrict__ tokens, int S, int m0,
                                                                  float *__restrict__ loss_rows, float scale) {
    __shared__ float red[256 / PHOTON_WAVE];
    constexpr int VEC = 16 / sizeof(T);
    typedef T vec_t __attribute__((ext_vector_type(VEC)));
    const int m = m0 + blockIdx.x;
    T *z = logits + (int64_t)blockIdx.x * ldz;
    const int tgt = tokens[(m / S) * (S + 1) + (m % S) + 1];
    const int nvec = V / VEC;
    vec_t v[NV];
    float mx = -INFINITY;
    // all loads first (a vector past the end re-reads vector 0 and is ignored below), so that they are in flight
    // together
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = threadIdx.x + 256 * j;
        v[j] = *reinterpret_cast<const vec_t *>(z + (i < nvec ? i : 0) * VEC);
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = threadIdx.x + 256 * j;
        if (i < nvec) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) mx = fmaxf(mx, to_f32(v[j][k]));
        }
    }
    for (int c = nvec * VEC + threadIdx.x; c < V; c += 256) mx = fmaxf(mx, to_f32(z[c]));
    const float gmx = block_max<256>(mx, red);
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = threadIdx.x + 256 * j;
        if (i < nvec) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) sum += __expf(to_f32(v[j][k]) - gmx);
        }
    }
    for (int c = nvec * VEC + threadIdx.x; c < V; c += 256) sum += __expf(to_f32(z[c]) - gmx);
    const float gsum = block_sum<256>(sum, red);
    const float lse = gmx + __logf(gsum);
    if (threadIdx.x == 0) loss_rows[m] = lse - to_f32(z[tgt]);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = threadIdx.x + 256 * j;
        if (i < nvec) {
            vec_t o;
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const int c = i * VEC + k;
                o[k] = from_f32<T>((__expf(to_f32(v[j][k]) - lse) - (c == tgt ? 1.0f : 0.0f)) * scale);
            }
            *reinterpret_cast<vec_t *>(z + i * VEC) = o;
        }
    }
    for (int c = nvec * VEC + threadIdx.x; c < ldz; c += 256) {
        float g = 0.f;
        if (c < V) g = (__expf(to_f32(z[c]) - lse) - (c == tgt ? 1.0f : 0.0f)) * scale;
        z[c] = from_f32<T>(g);
    }
}

__global__ __launch_bounds__(256) void loss_reduce_kernel(const float *__restrict__ rows, int M, double scale,
                                                           double *__restrict__ acc) {
    __shared__ double s[256];
    double a = 0.0;
    for (int i = threadIdx.x; i < M; i += 256) a += (double)rows[i];
    s[threadIdx.x] = a;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) acc[0] += s[0] * scale;
}

// ------------------------------------------------------------------------------------ misc

__global__ __launch_bounds__(256) void convert_bf16_kernel(const float *__restrict__ src, bf16 *__restrict__ dst,
                                                            int64_t n) {
    const int64_t nvec = n >> 3;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride) {
        const f32x4 a = *reinterpret_cast<const f32x4 *>(src + 8 * i);
        const f32x4 b = *reinterpret_cast<const f32x4 *>(src + 8 * i + 4);
        bf16x8 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            o[j] = (bf16)a[j];
            o[j + 4] = (bf16)b[j];
        }
        *reinterpret_cast<bf16x8 *>(dst + 8 * i) = o;
    }
    if (blockIdx.x == 0) {
        const int64_t i = (nvec << 3) + threadIdx.x;
        if (i < n) dst[i] = (bf16)src[i];
    }
}

// dst[c][r] = src[r][c] for a row-major [rows, cols] bf16 matrix, through a 64 x 64 LDS tile.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16 *__restrict__ src, bf16 *__restrict__ dst,
                                                              int rows, int cols) {
    __shared__ bf16 tile[64][64 + 2];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    for (int e = threadIdx.x; e < 64 * 64; e += 256) {
        const int r = e >> 6, c = e & 63;
        if (r0 + r < rows && c0 + c < cols) tile[r][c] = src[(int64_t)(r0 + r) * cols + c0 + c];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < 64 * 64; e += 256) {
        const int c = e >> 6, r = e & 63;
        if (r0 + r < rows && c0 + c < cols) dst[(int64_t)(c0 + c) * rows + r0 + r] = tile[r][c];
    }
}

// flag[0] = 1 if any id lies outside [0, V).  Every writer stores the same value, so plain
// stores suffice.
__global__ __launch_bounds__(256) void token_range_kernel(const int32_t *__restrict__ tok, int64_t n, int V,
                                                           int *__restrict__ flag) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    bool bad = false;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const int t = tok[i];
        bad |= (t < 0) | (t >= V);
    }
    if (bad) flag[0] = 1;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ p, int64_t n) {
    const int64_t nvec = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride)
        *reinterpret_cast<f32x4 *>(p + 4 * i) = f32x4{0.f, 0.f, 0.f, 0.f};
    if (blockIdx.x == 0) {
        const int64_t i = (nvec << 2) + threadIdx.x;
        if (i < n) p[i] = 0.f;
    }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// launchers

template <typename T>
void gemm_simple(hipStream_t st, GemmOp op, GemmEpi epi, const GemmArgs &g) {
    const dim3 grid((g.N + GT - 1) / GT, (g.M + GT - 1) / GT);
    if (op == GEMM_NN)
        hipLaunchKernelGGL((gemm_simple_kernel<T, GEMM_NN>), grid, dim3(256), 0, st, g, (int)epi);
    else if (op == GEMM_NT)
        hipLaunchKernelGGL((gemm_simple_kernel<T, GEMM_NT>), grid, dim3(256), 0, st, g, (int)epi);
    else
        hipLaunchKernelGGL((gemm_simple_kernel<T, GEMM_TN>), grid, dim3(256), 0, st, g, (int)epi);
}
template void gemm_simple<float>(hipStream_t, GemmOp, GemmEpi, const GemmArgs &);
template void gemm_simple<bf16>(hipStream_t, GemmOp, GemmEpi, const GemmArgs &);

template <>
void gemm<float>(hipStream_t st, GemmOp op, GemmEpi epi, const GemmArgs &g) {
    gemm_simple<float>(st, op, epi, g);
}
template <>
void gemm<bf16>(hipStream_t st, GemmOp op, GemmEpi epi, const GemmArgs &g) {
    TimedLaunch tl(st, KC_GEMM, 2.0 * (double)g.M * (double)g.N * (double)g.K);
    if (!gemm_mfma_bf16(st, op, epi, g)) gemm_simple<bf16>(st, op, epi, g);
}

template <>
void gemm_tn_accum_pair<float>(hipStream_t st, const GemmArgs &g1, const GemmArgs &g2) {
    gemm<float>(st, GEMM_TN, EPI_ACCUM, g1);
    gemm<float>(st, GEMM_TN, EPI_ACCUM, g2);
}
template <>
void gemm_tn_accum_pair<bf16>(hipStream_t st, const GemmArgs &g1, const GemmArgs &g2) {
    if (gemm_mfma_bf16_pair_covered(g1, g2)) {
        TimedLaunch tl(st, KC_GEMM, 2.0 * (double)g1.K * ((double)g1.M * (double)g1.N + (double)g2.M * (double)g2.N));
        gemm_mfma_bf16_pair_tn_accum(st, g1, g2);
        return;
    }
    gemm<bf16>(st, GEMM_TN, EPI_ACCUM, g1);
    gemm<bf16>(st, GEMM_TN, EPI_ACCUM, g2);
}

void embedding_gather(hipStream_t st, const float *E, const int32_t *tokens, float *x0, int B, int S, int d) {
    hipLaunchKernelGGL(embedding_gather_kernel, dim3(B * S), dim3(256), 0, st, E, tokens, x0, S, d);
}

void embedding_scatter_add(hipStream_t st, const float *dx0, const int32_t *tokens, float *dE, int B, int S, int d) {
    hipLaunchKernelGGL(embedding_scatter_kernel, dim3(B * S, (d + SCATTER_COLS - 1) / SCATTER_COLS), dim3(256), 0, st, dx0,
                       tokens, dE, S, B * S, d);
}

template <typename T>
void layernorm_fwd(hipStream_t st, const float *x, const float *gain, T *y, float *mean, float *rstd, int M, int d,
                   float eps) {
    const dim3 wgrid((M + 3) / 4), block(256);
    switch (d) {  // the widths of the model table: one wave per row
        case 768: hipLaunchKernelGGL((layernorm_fwd_wave_kernel<T, 3>), wgrid, block, 0, st, x, gain, y, mean, rstd, M, eps); return;
        case 1024: hipLaunchKernelGGL((layernorm_fwd_wave_kernel<T, 4>), wgrid, block, 0, st, x, gain, y, mean, rstd, M, eps); return;
        case 2048: hipLaunchKernelGGL((layernorm_fwd_wave_kernel<T, 8>), wgrid, block, 0, st, x, gain, y, mean, rstd, M, eps); return;
        case 2560: hipLaunchKernelGGL((layernorm_fwd_wave_kernel<T, 10>), wgrid, block, 0, st, x, gain, y, mean, rstd, M, eps); return;
        case 4096: hipLaunchKernelGGL((layernorm_fwd_wave_kernel<T, 16>), wgrid, block, 0, st, x, gain, y, mean, rstd, M, eps); return;
        default: break;
    }
    hipLaunchKernelGGL((layernorm_fwd_kernel<T>), dim3(M), dim3(LN_THREADS), 0, st, x, gain, y, mean, rstd, d, eps);
}
template void layernorm_fwd<float>(hipStream_t, const float *, const float *, float *, float *, float *, int, int, float);
template void layernorm_fwd<bf16>(hipStream_t, const float *, const float *, bf16 *, float *, float *, int, int, float);

constexpr int LN_BWD_BLOCKS = 512;
int layernorm_bwd_scratch_floats(int d) { return LN_BWD_BLOCKS * d; }

template <typename T, int NI>
static void launch_ln_bwd_wave(hipStream_t st, const T *dy, const float *x, const float *mean, const float *rstd,
                               const float *gain, const float *dres, float *dx_out, T *dx16, float *scratch, int M,
                               int blocks) {
    hipLaunchKernelGGL((layernorm_bwd_wave_kernel<T, NI>), dim3(blocks), dim3(256), 0, st, dy, x, mean, rstd, gain,
                       dres, dx_out, dx16, scratch, M);
}

template <typename T>
void layernorm_bwd(hipStream_t st, const T *dy, const float *x, const float *mean, const float *rstd,
                   const float *gain, const float *dres, float *dx_out, T *dx16, float *dgain, bool accumulate,
                   float *scratch, int M, int d) {
    int blocks = M < LN_BWD_BLOCKS ? M : LN_BWD_BLOCKS;
    bool wave_path = true;
    const int wblocks = (M + 3) / 4 < LN_BWD_BLOCKS ? (M + 3) / 4 : LN_BWD_BLOCKS;
    switch (d) {
        case 768: launch_ln_bwd_wave<T, 3>(st, dy, x, mean, rstd, gain, dres, dx_out, dx16, scratch, M, wblocks); break;
        case 1024: launch_ln_bwd_wave<T, 4>(st, dy, x, mean, rstd, gain, dres, dx_out, dx16, scratch, M, wblocks); break;
        case 2048: launch_ln_bwd_wave<T, 8>(st, dy, x, mean, rstd, gain, dres, dx_out, dx16, scratch, M, wblocks); break;
        case 2560: launch_ln_bwd_wave<T, 10>(st, dy, x, mean, rstd, gain, dres, dx_out, dx16, scratch, M, wblocks); break;
        case 4096: launch_ln_bwd_wave<T, 16>(st, dy, x, mean, rstd, gain, dres, dx_out, dx16, scratch, M, wblocks); break;
        default: wave_path = false; break;
    }
    if (wave_path) {
        blocks = wblocks;
    } else {
        hipLaunchKernelGGL((layernorm_bwd_kernel<T>), dim3(blocks), dim3(LN_THREADS), 0, st, dy, x, mean, rstd, gain,
                           dres, dx_out, dx16, scratch, M, d);
    }
    hipLaunchKernelGGL(colsum_accum_kernel, dim3((d + 15) / 16), dim3(256), 0, st, scratch, blocks, d, dgain,
                       accumulate);
}
template void layernorm_bwd<float>(hipStream_t, const float *, const float *, const float *, const float *,
                                   const float *, const float *, float *, float *, float *, bool, float *, int, int);
template void layernorm_bwd<bf16>(hipStream_t, const bf16 *, const float *, const float *, const float *,
                                  const float *, const float *, float *, bf16 *, float *, bool, float *, int, int);

template <typename T>
void attention_fwd_simple(hipStream_t st, const T *qkv, T *o, float *lse, int B, int H, int S, int Dh) {
    const size_t sm = sizeof(float) * (size_t)(S + Dh);
    hipLaunchKernelGGL((attn_fwd_simple_kernel<T>), dim3(S, H, B), dim3(64), sm, st, qkv, o, lse, H, S, Dh);
}
template void attention_fwd_simple<float>(hipStream_t, const float *, float *, float *, int, int, int, int);
template void attention_fwd_simple<bf16>(hipStream_t, const bf16 *, bf16 *, float *, int, int, int, int);

template <typename T>
void attention_bwd_simple(hipStream_t st, const T *qkv, const T *o, const float *lse, const T *d_o, T *dqkv,
                          float *dvec, int B, int H, int S, int Dh) {
    const size_t sm1 = sizeof(float) * (size_t)(S + 2 * Dh);
    hipLaunchKernelGGL((attn_bwd_dq_simple_kernel<T>), dim3(S, H, B), dim3(64), sm1, st, qkv, o, lse, d_o, dqkv, dvec, H,
                       S, Dh);
    const size_t sm2 = sizeof(float) * (size_t)(2 * S + 2 * Dh);
    hipLaunchKernelGGL((attn_bwd_dkv_simple_kernel<T>), dim3(S, H, B), dim3(64), sm2, st, qkv, lse, d_o, dqkv, dvec, H, S,
                       Dh);
}
template void attention_bwd_simple<float>(hipStream_t, const float *, const float *, const float *, const float *,
                                          float *, float *, int, int, int, int);
template void attention_bwd_simple<bf16>(hipStream_t, const bf16 *, const bf16 *, const float *, const bf16 *, bf16 *,
                                         float *, int, int, int, int);

template <>
void attention_fwd<float>(hipStream_t st, const float *qkv, float *o, float *lse, int B, int H, int S, int Dh) {
    attention_fwd_simple<float>(st, qkv, o, lse, B, H, S, Dh);
}
template <>
void attention_fwd<bf16>(hipStream_t st, const bf16 *qkv, bf16 *o, float *lse, int B, int H, int S, int Dh) {
    TimedLaunch tl(st, KC_ATTN, 2.0 * (double)B * H * (double)S * S * Dh);  // 4 S^2 Dh / 2 (causal)
    if (!attention_fwd_flash_bf16(st, qkv, o, lse, B, H, S, Dh)) attention_fwd_simple<bf16>(st, qkv, o, lse, B, H, S, Dh);
}
template <>
void attention_bwd<float>(hipStream_t st, const float *qkv, const float *o, const float *lse, const float *d_o,
                          float *dqkv, float *dvec, int B, int H, int S, int Dh) {
    attention_bwd_simple<float>(st, qkv, o, lse, d_o, dqkv, dvec, B, H, S, Dh);
}
template <>
void attention_bwd<bf16>(hipStream_t st, const bf16 *qkv, const bf16 *o, const float *lse, const bf16 *d_o, bf16 *dqkv,
                         float *dvec, int B, int H, int S, int Dh) {
    TimedLaunch tl(st, KC_ATTN, 5.0 * (double)B * H * (double)S * S * Dh);  // 10 S^2 Dh / 2 (causal)
    if (!attention_bwd_flash_bf16(st, qkv, o, lse, d_o, dqkv, dvec, B, H, S, Dh))
        attention_bwd_simple<bf16>(st, qkv, o, lse, d_o, dqkv, dvec, B, H, S, Dh);
}

template <typename T>
void cross_entropy_fwd_bwd(hipStream_t st, T *logits, int ldz, int V, const int32_t *tokens, int S, int m0, int rows,
                           float *loss_rows, float scale) {
    constexpr int VEC = 16 / sizeof(T), NV = 26;  // rows of up to 256 * 26 * VEC ids stay in registers
    if (V / VEC <= 256 * NV && sizeof(T) == 2)
        hipLaunchKernelGGL((cross_entropy_regs_kernel<T, NV>), dim3(rows), dim3(256), 0, st, logits, ldz, V, tokens, S, m0,
                           loss_rows, scale);
    else
        hipLaunchKernelGGL((cross_entropy_kernel<T>), dim3(rows), dim3(256), 0, st, logits, ldz, V, tokens, S, m0,
                           loss_rows, scale);
}
template void cross_entropy_fwd_bwd<float>(hipStream_t, float *, int, int, const int32_t *, int, int, int, float *, float);
template void cross_entropy_fwd_bwd<bf16>(hipStream_t, bf16 *, int, int, const int32_t *, int, int, int, float *, float);

void loss_reduce(hipStream_t st, const float *loss_rows, int M, double scale, double *acc) {
    hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(256), 0, st, loss_rows, M, scale, acc);
}

void convert_f32_to_bf16(hipStream_t st, const float *src, bf16 *dst, int64_t n) {
    hipLaunchKernelGGL(convert_bf16_kernel, dim3(2048), dim3(256), 0, st, src, dst, n);
}

void transpose_bf16(hipStream_t st, const bf16 *src, bf16 *dst, int rows, int cols) {
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((cols + 63) / 64, (rows + 63) / 64), dim3(256), 0, st, src, dst, rows,
                       cols);
}

void token_range_check(hipStream_t st, const int32_t *tokens, int64_t n, int V, int *flag) {
    fill_zero_f32(st, reinterpret_cast<float *>(flag), 1);
    const int64_t want = (n + 255) / 256;
    hipLaunchKernelGGL(token_range_kernel, dim3((unsigned)(want < 1024 ? (want > 0 ? want : 1) : 1024)), dim3(256), 0, st,
                       tokens, n, V, flag);
}

void fill_zero_f32(hipStream_t st, float *p, int64_t n) {
    const int64_t want = (n / 4 + 255) / 256 + 1;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)(want < 2048 ? want : 2048)), dim3(256), 0, st, p, n);
}
