// Bandwidth-bound kernels over flat parameter-length vectors: fused AdamW (ClientOpt of
// Alg. 3), pseudo-gradient export (Alg. 1: Delta_k = theta - theta_k), and the fused
// weighted-mean + server-optimizer pass (aggregator lines of Alg. 1, FedMom of the
// hyper-parameter appendix).
//
// All of them stream: every element is read once and written once, through 128-bit
// accesses that are contiguous across a wavefront, with a fixed grid (a multiple of the
// 256 compute units) walking the vector in grid strides.  Nothing uses atomics: sums of
// squares go to one fixed slot per workgroup and are combined in slot order in float64,
// so results are bit-identical between runs.

#include <cmath>
#include <mutex>
#include <vector>

#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kBlocks = 2048;  // 8 workgroups per compute unit; also the number of norm slots

__device__ __forceinline__ f32x4 ldg4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
__device__ __forceinline__ void stg4(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }

// ------------------------------------------------------------------------------------ AdamW

struct AdamScalars {
    float b1, b2, one_m_b1, one_m_b2, eps, decay /* 1 - lr*wd */, lr, inv_c1, inv_c2;
};

__device__ __forceinline__ void adam_elem(float &p, float &m, float &v, float g, const AdamScalars &s) {
    m = s.b1 * m + s.one_m_b1 * g;
    v = s.b2 * v + s.one_m_b2 * (g * g);
    const float mhat = m * s.inv_c1;
    const float vhat = v * s.inv_c2;
    p = p * s.decay - s.lr * (mhat / (sqrtf(vhat) + s.eps));
}

template <bool W16>
__global__ __launch_bounds__(kThreads) void adamw_kernel(float *__restrict__ p, float *__restrict__ m,
                                                          float *__restrict__ v, const float *__restrict__ g,
                                                          bf16 *__restrict__ w16, int64_t n, AdamScalars s) {
    const int64_t nvec = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
        f32x4 pp = ldg4(p + 4 * i), mm = ldg4(m + 4 * i), vv = ldg4(v + 4 * i), gg = ldg4(g + 4 * i);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float pj = pp[j], mj = mm[j], vj = vv[j];
            adam_elem(pj, mj, vj, gg[j], s);
            pp[j] = pj;
            mm[j] = mj;
            vv[j] = vj;
        }
        stg4(p + 4 * i, pp);
        stg4(m + 4 * i, mm);
        stg4(v + 4 * i, vv);
        if constexpr (W16) {
            bf16x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = (bf16)pp[j];
            *reinterpret_cast<bf16x4 *>(w16 + 4 * i) = o;
        }
    }
    // ragged tail (n % 4 elements), one thread each
    if (blockIdx.x == 0) {
        const int64_t i = (nvec << 2) + threadIdx.x;
        if (i < n) {
            float pp = p[i], mm = m[i], vv = v[i];
            adam_elem(pp, mm, vv, g[i], s);
            p[i] = pp;
            m[i] = mm;
            v[i] = vv;
            if constexpr (W16) w16[i] = (bf16)pp;
        }
    }
}

// AdamW over a set of row-major matrices of the flat vector, 64 x 64 tiles, writing besides the
// updated parameters and moments the bf16 working copy (same layout) and its transpose
// ([cols, rows] at the same offset of w16t) in the same pass: the forward products read the
// transposed weights, and a separate transpose pass after every optimizer step would read and
// write the whole bf16 copy once more.  A tile's rows are read and written as 256-byte row pieces;
// the transposed tile goes through LDS so that its rows are written as 128-byte pieces.
constexpr int AT = 64;  // tile edge
struct AdamMatrix {
    int64_t offset;      // first element in the flat vector
    int rows, cols;
    int tile_begin;      // index of the matrix's first tile among all tiles
};
__global__ __launch_bounds__(kThreads) void adamw_tiles_kernel(float *__restrict__ p, float *__restrict__ m,
                                                                float *__restrict__ v, const float *__restrict__ g,
                                                                bf16 *__restrict__ w16, bf16 *__restrict__ w16t,
                                                                const AdamMatrix *__restrict__ mats, int n_mats,
                                                                int n_tiles, AdamScalars s) {
    __shared__ bf16 tile[AT][AT + 2];
    for (int tix = blockIdx.x; tix < n_tiles; tix += gridDim.x) {
        // the matrix this tile belongs to: tile_begin is increasing, a handful of entries per block
        int lo = 0, hi = n_mats - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (mats[mid].tile_begin <= tix) lo = mid;
            else hi = mid - 1;
        }
        const AdamMatrix mt = mats[lo];
        const int tiles_c = (mt.cols + AT - 1) / AT;
        const int r0 = ((tix - mt.tile_begin) / tiles_c) * AT, c0 = ((tix - mt.tile_begin) % tiles_c) * AT;
        const int cq = (threadIdx.x & 15) * 4, rq = threadIdx.x >> 4;  // 4 columns, rows rq, rq + 16, ..
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int r = rq + 16 * k;
            if (r0 + r < mt.rows && c0 + cq < mt.cols) {  // cols % 4 == 0: a quad is inside or outside as a whole
                const int64_t i = mt.offset + (int64_t)(r0 + r) * mt.cols + c0 + cq;
                f32x4 pp = ldg4(p + i), mm = ldg4(m + i), vv = ldg4(v + i), gg = ldg4(g + i);
                bf16x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float pj = pp[j], mj = mm[j], vj = vv[j];
                    adam_elem(pj, mj, vj, gg[j], s);
                    pp[j] = pj;
                    mm[j] = mj;
                    vv[j] = vj;
                    o[j] = (bf16)pj;
                    tile[r][cq + j] = o[j];
                }
                stg4(p + i, pp);
                stg4(m + i, mm);
                stg4(v + i, vv);
                *reinterpret_cast<bf16x4 *>(w16 + i) = o;
            }
        }
        __syncthreads();
        // transposed tile: row c of it = column c0 + c of the matrix, rows r0 .. r0 + 63
        const int tr4 = (threadIdx.x & 15) * 4, tc = threadIdx.x >> 4;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int cc = tc + 16 * k;
            if (c0 + cc < mt.cols && r0 + tr4 < mt.rows) {
                bf16 *dst = w16t + mt.offset + (int64_t)(c0 + cc) * mt.rows + r0 + tr4;
                if (mt.rows % 4 == 0) {
                    bf16x4 o;
#pragma unroll
                    for (int j = 0; j < 4; ++j) o[j] = tile[tr4 + j][cc];
                    *reinterpret_cast<bf16x4 *>(dst) = o;
                } else {
                    for (int j = 0; j < 4 && r0 + tr4 + j < mt.rows; ++j) dst[j] = tile[tr4 + j][cc];
                }
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------ client init

// client <- global, m <- 0, v <- 0 in one pass (4 B read, 12 B written per parameter)
__global__ __launch_bounds__(kThreads) void client_init_kernel(const float *__restrict__ gl, float *__restrict__ cl,
                                                                float *__restrict__ m, float *__restrict__ v,
                                                                int64_t n) {
    const int64_t nvec = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
        stg4(cl + 4 * i, ldg4(gl + 4 * i));
        stg4(m + 4 * i, z);
        stg4(v + 4 * i, z);
    }
    if (blockIdx.x == 0) {
        const int64_t i = (nvec << 2) + threadIdx.x;
        if (i < n) {
            cl[i] = gl[i];
            m[i] = 0.f;
            v[i] = 0.f;
        }
    }
}

// ------------------------------------------------------------------------------------ delta export

template <typename T>
__global__ __launch_bounds__(kThreads) void export_delta_kernel(const float *__restrict__ gl,
                                                                 const float *__restrict__ cl, T *__restrict__ out,
                                                                 int64_t n) {
    const int64_t nvec = n >> 3;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
        const f32x4 a0 = ldg4(gl + 8 * i), a1 = ldg4(gl + 8 * i + 4);
        const f32x4 c0 = ldg4(cl + 8 * i), c1 = ldg4(cl + 8 * i + 4);
        if constexpr (sizeof(T) == 2) {
            bf16x8 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o[j] = (bf16)(a0[j] - c0[j]);
                o[j + 4] = (bf16)(a1[j] - c1[j]);
            }
            *reinterpret_cast<bf16x8 *>(out + 8 * i) = o;
        } else {
            stg4(reinterpret_cast<float *>(out) + 8 * i, a0 - c0);
            stg4(reinterpret_cast<float *>(out) + 8 * i + 4, a1 - c1);
        }
    }
    if (blockIdx.x == 0) {
        const int64_t i = (nvec << 3) + threadIdx.x;
        if (i < n) out[i] = from_f32<T>(gl[i] - cl[i]);
    }
}

// ------------------------------------------------------------------------------------ aggregation

constexpr int KIND_PARAMS_F32 = 0, KIND_DELTA_F32 = 1, KIND_DELTA_BF16 = 2;

struct ClientArgs {
    const void *ptr[PHOTON_MAX_CLIENTS];
    float w[PHOTON_MAX_CLIENTS];  // normalised weights
};

struct OuterScalars {
    float eta, mu;
    int nesterov;
};

// Eight consecutive pseudo-gradient values of client buffer `base` at vector index i.
template <int KIND>
__device__ __forceinline__ void load_delta8(const void *base, int64_t i, const float (&th)[8], float (&d)[8]) {
    if constexpr (KIND == KIND_DELTA_BF16) {
        const bf16x8 r = *reinterpret_cast<const bf16x8 *>(reinterpret_cast<const bf16 *>(base) + 8 * i);
#pragma unroll
        for (int j = 0; j < 8; ++j) d[j] = (float)r[j];
    } else {
        const float *fp = reinterpret_cast<const float *>(base) + 8 * i;
        const f32x4 r0 = ldg4(fp), r1 = ldg4(fp + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            d[j] = r0[j];
            d[j + 4] = r1[j];
        }
        if constexpr (KIND == KIND_PARAMS_F32) {
#pragma unroll
            for (int j = 0; j < 8; ++j) d[j] = th[j] - d[j];
        }
    }
}

template <int KIND>
__device__ __forceinline__ float load_delta1(const void *base, int64_t i, float th) {
    if constexpr (KIND == KIND_DELTA_BF16) return (float)reinterpret_cast<const bf16 *>(base)[i];
    const float r = reinterpret_cast<const float *>(base)[i];
    return KIND == KIND_PARAMS_F32 ? th - r : r;
}

__device__ __forceinline__ float outer_elem(float th, float delta, float &b, const OuterScalars &o, bool mom) {
    float u = delta;
    if (mom) {
        b = o.mu * b + delta;
        u = o.nesterov ? delta + o.mu * b : b;
    }
    return th - o.eta * u;
}

// KT > 0: exactly KT clients, register accumulators, per-client norms.  KT == 0: run-time K
// (no per-client norms; sumsq_kernel takes them beforehand when they are asked for).
template <int KIND, int KT, bool MOM>
__global__ __launch_bounds__(kThreads) void aggregate_kernel(float *__restrict__ theta, float *__restrict__ mom,
                                                              ClientArgs ca, int K, OuterScalars os, int64_t n,
                                                              float *__restrict__ partials) {
    constexpr int NK = KT > 0 ? KT : 1;
    __shared__ float red[kThreads / PHOTON_WAVE];
    const int64_t nvec = n >> 3;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    double nd = 0.0;
    double nk[NK];
#pragma unroll
    for (int k = 0; k < NK; ++k) nk[k] = 0.0;

    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
        float th[8], b[8], acc[8];
        {
            const f32x4 t0 = ldg4(theta + 8 * i), t1 = ldg4(theta + 8 * i + 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                th[j] = t0[j];
                th[j + 4] = t1[j];
            }
        }
        if constexpr (MOM) {
            const f32x4 b0 = ldg4(mom + 8 * i), b1 = ldg4(mom + 8 * i + 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                b[j] = b0[j];
                b[j + 4] = b1[j];
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;

        if constexpr (KT > 0) {
            float d[KT][8];
#pragma unroll
            for (int k = 0; k < KT; ++k) load_delta8<KIND>(ca.ptr[k], i, th, d[k]);
#pragma unroll
            for (int k = 0; k < KT; ++k) {  // fixed order k = 0 .. K-1, one FMA per term
                float sq = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    acc[j] = fmaf(ca.w[k], d[k][j], acc[j]);
                    sq = fmaf(d[k][j], d[k][j], sq);
                }
                nk[k] += (double)sq;
            }
        } else {
            for (int k = 0; k < K; ++k) {
                float d[8];
                load_delta8<KIND>(ca.ptr[k], i, th, d);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = fmaf(ca.w[k], d[j], acc[j]);
            }
        }
        float sq = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            sq = fmaf(acc[j], acc[j], sq);
            th[j] = outer_elem(th[j], acc[j], b[j], os, MOM);
        }
        nd += (double)sq;
        stg4(theta + 8 * i, f32x4{th[0], th[1], th[2], th[3]});
        stg4(theta + 8 * i + 4, f32x4{th[4], th[5], th[6], th[7]});
        if constexpr (MOM) {
            stg4(mom + 8 * i, f32x4{b[0], b[1], b[2], b[3]});
            stg4(mom + 8 * i + 4, f32x4{b[4], b[5], b[6], b[7]});
        }
    }
    // ragged tail (n % 8 elements)
    if (blockIdx.x == 0) {
        const int64_t i = (nvec << 3) + threadIdx.x;
        if (i < n) {
            float th = theta[i], b = MOM ? mom[i] : 0.f, acc = 0.f;
            if constexpr (KT > 0) {
#pragma unroll
                for (int k = 0; k < KT; ++k) {
                    const float d = load_delta1<KIND>(ca.ptr[k], i, th);
                    acc = fmaf(ca.w[k], d, acc);
                    nk[k] += (double)(d * d);
                }
            } else {
                for (int k = 0; k < K; ++k) acc = fmaf(ca.w[k], load_delta1<KIND>(ca.ptr[k], i, th), acc);
            }
            nd += (double)(acc * acc);
            theta[i] = outer_elem(th, acc, b, os, MOM);
            if constexpr (MOM) mom[i] = b;
        }
    }
    // one slot per workgroup and quantity; float32 slots of float64-accumulated thread sums
    const float sd = block_sum<kThreads>((float)nd, red);
    if (threadIdx.x == 0) partials[blockIdx.x] = sd;
    if constexpr (KT > 0) {
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            const float sk = block_sum<kThreads>((float)nk[k], red);
            if (threadIdx.x == 0) partials[(int64_t)(k + 1) * gridDim.x + blockIdx.x] = sk;
        }
    }
}

// Sum of squares of one client's pseudo-gradient into its row of slots: the buffer itself
// (KIND = deltas) or theta - buffer (KIND = client parameters).
template <int KIND>
__global__ __launch_bounds__(kThreads) void sumsq_kernel(const void *__restrict__ x, const float *__restrict__ theta,
                                                          int64_t n, float *__restrict__ partials) {
    __shared__ float red[kThreads / PHOTON_WAVE];
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    double acc = 0.0;
    const int64_t nvec = n >> 3;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
        float d[8], th[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if constexpr (KIND == KIND_PARAMS_F32) {
            const f32x4 t0 = ldg4(theta + 8 * i), t1 = ldg4(theta + 8 * i + 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                th[j] = t0[j];
                th[j + 4] = t1[j];
            }
        }
        load_delta8<KIND>(x, i, th, d);
        float sq = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) sq = fmaf(d[j], d[j], sq);
        acc += (double)sq;
    }
    if (blockIdx.x == 0) {
        const int64_t i = (nvec << 3) + threadIdx.x;
        if (i < n) {
            const float d = load_delta1<KIND>(x, i, KIND == KIND_PARAMS_F32 ? theta[i] : 0.f);
            acc += (double)(d * d);
        }
    }
    const float s = block_sum<kThreads>((float)acc, red);
    if (threadIdx.x == 0) partials[blockIdx.x] = s;
}

// Row r of the slots -> out[r], float64, fixed order.
__global__ __launch_bounds__(kThreads) void finish_norms_kernel(const float *__restrict__ partials, int nslots,
                                                                 double *__restrict__ out) {
    __shared__ double s[kThreads];
    const float *row = partials + (int64_t)blockIdx.x * nslots;
    double acc = 0.0;
    for (int i = threadIdx.x; i < nslots; i += kThreads) acc += (double)row[i];
    s[threadIdx.x] = acc;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[blockIdx.x] = s[0];
}

// delta *= min(1, max_norm / sqrt(norm2[0]))
template <typename T>
__global__ __launch_bounds__(kThreads) void clip_scale_kernel(T *__restrict__ x, int64_t n,
                                                               const double *__restrict__ norm2, double max_norm) {
    const double nrm = sqrt(norm2[0]);
    if (!(nrm > max_norm)) return;
    const float sc = (float)(max_norm / nrm);
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
        x[i] = from_f32<T>(to_f32(x[i]) * sc);
}

template <int KIND, int KT>
void launch_aggregate(bool mom, hipStream_t st, float *theta, float *mb, const ClientArgs &ca, int K,
                      OuterScalars os, int64_t n, float *partials) {
    if (mom)
        hipLaunchKernelGGL((aggregate_kernel<KIND, KT, true>), dim3(kBlocks), dim3(kThreads), 0, st, theta, mb, ca, K,
                           os, n, partials);
    else
        hipLaunchKernelGGL((aggregate_kernel<KIND, KT, false>), dim3(kBlocks), dim3(kThreads), 0, st, theta, mb, ca,
                           K, os, n, partials);
}

template <int KIND>
void dispatch_aggregate(bool mom, hipStream_t st, float *theta, float *mb, const ClientArgs &ca, int K,
                        OuterScalars os, int64_t n, float *partials) {
    switch (K) {
        case 1: launch_aggregate<KIND, 1>(mom, st, theta, mb, ca, K, os, n, partials); break;
        case 2: launch_aggregate<KIND, 2>(mom, st, theta, mb, ca, K, os, n, partials); break;
        case 3: launch_aggregate<KIND, 3>(mom, st, theta, mb, ca, K, os, n, partials); break;
        case 4: launch_aggregate<KIND, 4>(mom, st, theta, mb, ca, K, os, n, partials); break;
        case 5: launch_aggregate<KIND, 5>(mom, st, theta, mb, ca, K, os, n, partials); break;
        case 6: launch_aggregate<KIND, 6>(mom, st, theta, mb, ca, K, os, n, partials); break;
        case 7: launch_aggregate<KIND, 7>(mom, st, theta, mb, ca, K, os, n, partials); break;
        case 8: launch_aggregate<KIND, 8>(mom, st, theta, mb, ca, K, os, n, partials); break;
        default: launch_aggregate<KIND, 0>(mom, st, theta, mb, ca, K, os, n, partials); break;
    }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// host side

int flat_init(photon_ctx *ctx) {
    ctx->norm_blocks = kBlocks;
    const size_t pbytes = sizeof(float) * (size_t)(PHOTON_MAX_CLIENTS + 1) * kBlocks;
    if (hipMalloc(&ctx->norm_partials, pbytes) != hipSuccess) return PHOTON_ENOMEM;
    if (hipMalloc(&ctx->norm_out, sizeof(double) * (PHOTON_MAX_CLIENTS + 1)) != hipSuccess) return PHOTON_ENOMEM;
    if (hipHostMalloc(&ctx->norm_host, sizeof(double) * (PHOTON_MAX_CLIENTS + 1), hipHostMallocDefault) != hipSuccess)
        return PHOTON_ENOMEM;
    ctx->workspace_bytes += (int64_t)pbytes + (int64_t)sizeof(double) * (PHOTON_MAX_CLIENTS + 1);
    return PHOTON_OK;
}

void flat_free(photon_ctx *ctx) {
    if (ctx->norm_partials) (void)hipFree(ctx->norm_partials);
    if (ctx->norm_out) (void)hipFree(ctx->norm_out);
    if (ctx->norm_host) (void)hipHostFree(ctx->norm_host);
    ctx->norm_partials = nullptr;
    ctx->norm_out = nullptr;
    ctx->norm_host = nullptr;
}

static AdamScalars adam_scalars(int64_t t, float lr, const photon_adamw_hp *hp);

int flat_adamw(photon_ctx *ctx, float *p, float *m, float *v, const float *g, int64_t n, int64_t t, float lr,
               const photon_adamw_hp *hp, bf16 *w16) {
    const AdamScalars s = adam_scalars(t, lr, hp);
    TimedLaunch tl(ctx->stream, KC_ADAMW, (double)n * (w16 ? 30.0 : 28.0));
    if (w16)
        hipLaunchKernelGGL((adamw_kernel<true>), dim3(kBlocks), dim3(kThreads), 0, ctx->stream, p, m, v, g, w16, n, s);
    else
        hipLaunchKernelGGL((adamw_kernel<false>), dim3(kBlocks), dim3(kThreads), 0, ctx->stream, p, m, v, g, w16, n, s);
    HIP_TRY(ctx, hipGetLastError());
    return PHOTON_OK;
}

static AdamScalars adam_scalars(int64_t t, float lr, const photon_adamw_hp *hp) {
    AdamScalars s;
    s.b1 = hp->beta1;
    s.b2 = hp->beta2;
    s.one_m_b1 = 1.0f - hp->beta1;
    s.one_m_b2 = 1.0f - hp->beta2;
    s.eps = hp->eps;
    s.lr = lr;
    s.decay = (float)(1.0 - (double)lr * (double)hp->weight_decay);
    s.inv_c1 = (float)(1.0 / (1.0 - pow((double)hp->beta1, (double)t)));
    s.inv_c2 = (float)(1.0 / (1.0 - pow((double)hp->beta2, (double)t)));
    return s;
}

// The matrices of the flat vector as the tiled kernel wants them (device table, built once).
int flat_adamw_table(photon_ctx *ctx, const int64_t *offsets, const int *rows, const int *cols, int n_mats,
                     void **table_out, int *tiles_out) {
    std::vector<AdamMatrix> host(n_mats);
    int tiles = 0;
    for (int i = 0; i < n_mats; ++i) {
        host[i] = AdamMatrix{offsets[i], rows[i], cols[i], tiles};
        tiles += ((rows[i] + AT - 1) / AT) * ((cols[i] + AT - 1) / AT);
    }
    void *dev = nullptr;
    if (hipMalloc(&dev, sizeof(AdamMatrix) * (size_t)n_mats) != hipSuccess) return PHOTON_ENOMEM;
    HIP_TRY(ctx, hipMemcpy(dev, host.data(), sizeof(AdamMatrix) * (size_t)n_mats, hipMemcpyHostToDevice));
    *table_out = dev;
    *tiles_out = tiles;
    return PHOTON_OK;
}

int flat_adamw_tiled(photon_ctx *ctx, float *p, float *m, float *v, const float *g, int64_t n, int64_t t, float lr,
                     const photon_adamw_hp *hp, bf16 *w16, bf16 *w16t, const void *table, int n_mats, int n_tiles) {
    const AdamScalars s = adam_scalars(t, lr, hp);
    TimedLaunch tl(ctx->stream, KC_ADAMW, (double)n * 32.0);  // 16 B read, 12 + 2 + 2 B written per parameter
    const int grid = n_tiles < 16 * kBlocks ? n_tiles : 16 * kBlocks;
    hipLaunchKernelGGL(adamw_tiles_kernel, dim3(grid), dim3(kThreads), 0, ctx->stream, p, m, v, g, w16, w16t,
                       (const AdamMatrix *)table, n_mats, n_tiles, s);
    HIP_TRY(ctx, hipGetLastError());
    return PHOTON_OK;
}

int flat_client_init(photon_ctx *ctx, const float *gl, float *cl, float *m, float *v, int64_t n) {
    hipLaunchKernelGGL(client_init_kernel, dim3(kBlocks), dim3(kThreads), 0, ctx->stream, gl, cl, m, v, n);
    HIP_TRY(ctx, hipGetLastError());
    return PHOTON_OK;
}

int flat_export_delta(photon_ctx *ctx, const float *gl, const float *cl, void *out, int dtype, int64_t n) {
    TimedLaunch tl(ctx->stream, KC_DELTA, (double)n * (dtype == PHOTON_BF16 ? 10.0 : 12.0));
    if (dtype == PHOTON_BF16)
        hipLaunchKernelGGL((export_delta_kernel<bf16>), dim3(kBlocks), dim3(kThreads), 0, ctx->stream, gl, cl,
                           (bf16 *)out, n);
    else
        hipLaunchKernelGGL((export_delta_kernel<float>), dim3(kBlocks), dim3(kThreads), 0, ctx->stream, gl, cl,
                           (float *)out, n);
    HIP_TRY(ctx, hipGetLastError());
    return PHOTON_OK;
}

// Kernel launches of one aggregation on `st`: the fused weighted sum + server step, and, when
// norms_dev is given, the squared norms (averaged pseudo-gradient first, then the K clients')
// as float64 in norms_dev[0 .. K].  `part` holds (K + 1) rows of kBlocks slots; every slot that is
// read is written first by this call.  Nothing here allocates or synchronises.
static void aggregate_launches(hipStream_t st, float *global, const void *const *bufs, int K, int kind, int dtype,
                               const float *wnorm, const photon_outer_opt *oo, int64_t n, float *part,
                               double *norms_dev) {
    ClientArgs ca{};
    for (int k = 0; k < K; ++k) {
        ca.ptr[k] = bufs[k];
        ca.w[k] = wnorm[k];
    }
    const OuterScalars os{oo->eta_s, oo->mu, oo->nesterov};
    const bool mom = oo->mu != 0.0f;
    const int kk = kind == PHOTON_CLIENT_PARAMS ? KIND_PARAMS_F32 : dtype == PHOTON_FP32 ? KIND_DELTA_F32 : KIND_DELTA_BF16;
    if (norms_dev && K > 8) {
        // the run-time-K kernel takes no per-client norms: one pass per client, before the global
        // model moves (client parameters are turned into pseudo-gradients against the old model)
        for (int k = 0; k < K; ++k) {
            float *row = part + (int64_t)(k + 1) * kBlocks;
            if (kk == KIND_PARAMS_F32)
                hipLaunchKernelGGL((sumsq_kernel<KIND_PARAMS_F32>), dim3(kBlocks), dim3(kThreads), 0, st, bufs[k], global, n, row);
            else if (kk == KIND_DELTA_F32)
                hipLaunchKernelGGL((sumsq_kernel<KIND_DELTA_F32>), dim3(kBlocks), dim3(kThreads), 0, st, bufs[k], global, n, row);
            else
                hipLaunchKernelGGL((sumsq_kernel<KIND_DELTA_BF16>), dim3(kBlocks), dim3(kThreads), 0, st, bufs[k], global, n, row);
        }
    }
    {
        const double client_b = kk == KIND_DELTA_BF16 ? 2.0 : 4.0;
        TimedLaunch tl(st, KC_AGG, (double)n * (client_b * K + 8.0 + (mom ? 8.0 : 0.0)));
        if (kk == KIND_PARAMS_F32)
            dispatch_aggregate<KIND_PARAMS_F32>(mom, st, global, oo->momentum, ca, K, os, n, part);
        else if (kk == KIND_DELTA_F32)
            dispatch_aggregate<KIND_DELTA_F32>(mom, st, global, oo->momentum, ca, K, os, n, part);
        else
            dispatch_aggregate<KIND_DELTA_BF16>(mom, st, global, oo->momentum, ca, K, os, n, part);
    }
    if (norms_dev)
        hipLaunchKernelGGL(finish_norms_kernel, dim3(K + 1), dim3(kThreads), 0, st, part, kBlocks, norms_dev);
}

int flat_aggregate(photon_ctx *ctx, float *global, const void *const *bufs, int K, int kind, int dtype,
                   const float *wnorm, photon_outer_opt *oo, photon_agg_metrics *metrics, int64_t n) {
    hipStream_t st = ctx->stream;
    aggregate_launches(st, global, bufs, K, kind, dtype, wnorm, oo, n, ctx->norm_partials,
                       metrics ? ctx->norm_out : nullptr);
    HIP_TRY(ctx, hipGetLastError());
    oo->round += 1;
    if (!metrics) return PHOTON_OK;
    HIP_TRY(ctx, hipMemcpyAsync(ctx->norm_host, ctx->norm_out, sizeof(double) * (K + 1), hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    metrics->delta_norm2 = ctx->norm_host[0];
    for (int k = 0; k < PHOTON_MAX_CLIENTS; ++k) metrics->client_norm2[k] = k < K ? ctx->norm_host[k + 1] : 0.0;
    return PHOTON_OK;
}

// ---------------------------------------------------------------------------------------------
// Aggregation without a context and without any allocation: the norm slots live in a file-scope
// device array instead of the context's workspace.  Each GPU holds its own copy of the array at
// its own address; the address is looked up once per device, with that device current, and only
// that pointer is ever handed to kernels (the array's name is a host-side stand-in in host code).

static __device__ __align__(256) float scratch[(PHOTON_STATIC_MAX_CLIENTS + 1) * kBlocks];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float *g_scratch_ptr[kMaxDevices] = {};

// device pointer of `scratch` on the current device; nullptr (and *err set) on failure
float *scratch_on_current_device(hipError_t *err) {
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = static_cast<float *>(p);
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int flat_aggregate_static(hipStream_t st, float *global, const void *const *bufs, int K, int kind, int dtype,
                          const float *wnorm, photon_outer_opt *oo, double *norms_dev, int64_t n, int *hip_error) {
    hipError_t e = hipSuccess;
    float *part = scratch_on_current_device(&e);
    if (!part) {
        if (hip_error) *hip_error = (int)e;
        return PHOTON_EHIP;
    }
    aggregate_launches(st, global, bufs, K, kind, dtype, wnorm, oo, n, part, norms_dev);
    e = hipGetLastError();
    if (e != hipSuccess) {
        if (hip_error) *hip_error = (int)e;
        return PHOTON_EHIP;
    }
    oo->round += 1;
    return PHOTON_OK;
}

int flat_clip(photon_ctx *ctx, void *delta, int dtype, double max_norm, double *norm_out, int64_t n) {
    hipStream_t st = ctx->stream;
    const float *none = nullptr;
    if (dtype == PHOTON_BF16)
        hipLaunchKernelGGL((sumsq_kernel<KIND_DELTA_BF16>), dim3(kBlocks), dim3(kThreads), 0, st, (const void *)delta, none, n,
                           ctx->norm_partials);
    else
        hipLaunchKernelGGL((sumsq_kernel<KIND_DELTA_F32>), dim3(kBlocks), dim3(kThreads), 0, st, (const void *)delta, none, n,
                           ctx->norm_partials);
    hipLaunchKernelGGL(finish_norms_kernel, dim3(1), dim3(kThreads), 0, st, ctx->norm_partials, kBlocks, ctx->norm_out);
    if (dtype == PHOTON_BF16)
        hipLaunchKernelGGL((clip_scale_kernel<bf16>), dim3(kBlocks), dim3(kThreads), 0, st, (bf16 *)delta, n,
                           ctx->norm_out, max_norm);
    else
        hipLaunchKernelGGL((clip_scale_kernel<float>), dim3(kBlocks), dim3(kThreads), 0, st, (float *)delta, n,
                           ctx->norm_out, max_norm);
    HIP_TRY(ctx, hipGetLastError());
    if (norm_out) {
        HIP_TRY(ctx, hipMemcpyAsync(ctx->norm_host, ctx->norm_out, sizeof(double), hipMemcpyDeviceToHost, st));
        HIP_TRY(ctx, hipStreamSynchronize(st));
        *norm_out = sqrt(ctx->norm_host[0]);
    }
    return PHOTON_OK;
}
