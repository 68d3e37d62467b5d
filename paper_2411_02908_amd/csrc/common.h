// Internal declarations shared by the translation units of libphoton (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <vector>

#include "photon.h"

typedef __bf16 bf16;
typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define PHOTON_WAVE 64

// ---------------------------------------------------------------------------------------------
// context

struct ModelWorkspace;  // model.hip

// Per-kernel-class event timing (profile.hip).
enum KernelClass { KC_GEMM = 0, KC_ATTN, KC_ADAMW, KC_AGG, KC_DELTA, KC_COUNT };
struct KernelTimer {
    bool on = false;
    int every = 1;                 // GEMM and attention classes: time every `every`-th launch
    int64_t seen[KC_COUNT] = {};   // launches of each class since timing began, timed or not
    std::vector<hipEvent_t> pool;
    size_t used = 0;
    struct Rec {
        int cls;
        double work;
        size_t e0, e1;
    };
    std::vector<Rec> recs;
};
extern thread_local KernelTimer *g_timer;  // set while an API call of a profiling ctx runs
struct TimedLaunch {                       // RAII: events around the launches in its scope
    hipStream_t st;
    size_t rec;
    bool active;
    TimedLaunch(hipStream_t stream, int cls, double work);
    ~TimedLaunch();
};
struct TimerScope {  // binds g_timer for the duration of an API call
    explicit TimerScope(struct photon_ctx *ctx);
    ~TimerScope();
};

struct photon_ctx {
    hipStream_t stream = nullptr;
    int64_t n = 0;                 // flat vector length
    int last_hip_error = 0;
    int64_t workspace_bytes = 0;
    // flat-vector scratch: per-block partial sums of squares, fixed slots
    float *norm_partials = nullptr;   // [(PHOTON_MAX_CLIENTS + 1)][norm_blocks]
    double *norm_out = nullptr;       // [(PHOTON_MAX_CLIENTS + 1)] device
    double *norm_host = nullptr;      // pinned mirror
    int norm_blocks = 0;
    bool has_model = false;
    photon_model_cfg cfg{};
    int micro_batch = 0;
    ModelWorkspace *ws = nullptr;
    KernelTimer timer;
};

#define HIP_TRY(ctx, expr)                                   \
    do {                                                     \
        hipError_t e_ = (expr);                              \
        if (e_ != hipSuccess) {                              \
            (ctx)->last_hip_error = (int)e_;                 \
            return PHOTON_EHIP;                              \
        }                                                    \
    } while (0)

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---------------------------------------------------------------------------------------------
// device helpers

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// Block-wide sum in a fixed order (lanes by butterfly, then waves 0..nw-1); result on all threads.
template <int THREADS>
__device__ __forceinline__ float block_sum(float v, float *smem /* >= THREADS/64 floats */) {
    constexpr int NW = THREADS / PHOTON_WAVE;
    v = wave_sum(v);
    if constexpr (NW == 1) return v;
    const int w = threadIdx.x / PHOTON_WAVE;
    __syncthreads();
    if ((threadIdx.x & (PHOTON_WAVE - 1)) == 0) smem[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) t += smem[i];
    return t;
}

template <int THREADS>
__device__ __forceinline__ float block_max(float v, float *smem) {
    constexpr int NW = THREADS / PHOTON_WAVE;
    v = wave_max(v);
    if constexpr (NW == 1) return v;
    const int w = threadIdx.x / PHOTON_WAVE;
    __syncthreads();
    if ((threadIdx.x & (PHOTON_WAVE - 1)) == 0) smem[w] = v;
    __syncthreads();
    float t = smem[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) t = fmaxf(t, smem[i]);
    return t;
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return (float)x; }
template <typename T>
__device__ __forceinline__ T from_f32(float x);
template <>
__device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <>
__device__ __forceinline__ bf16 from_f32<bf16>(float x) { return (bf16)x; }  // v_cvt_pk_bf16_f32: RNE

// ---------------------------------------------------------------------------------------------
// Global -> LDS copies (buffer_load ... lds) and LDS transpose reads.

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef int rsrc_t __attribute__((ext_vector_type(4)));

// Buffer descriptor of `bytes` bytes at p: loads past the end return zero, which is what ragged
// last tiles need.  Words: base address (48 bits, stride 0), size in bytes, raw-buffer format.
__device__ __forceinline__ rsrc_t make_rsrc(const void *p, uint32_t bytes) {
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    return rsrc_t{(int)(uint32_t)a, (int)(uint32_t)((a >> 32) & 0xffffu), (int)bytes, 0x00020000};
}

__device__ __forceinline__ unsigned lds_addr(const void *p) {
    return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char *)(p);
}

// Copy of 16 (resp. 4) bytes per lane from global memory straight into LDS at
// lds_byte_addr + 16 (resp. 4) * lane, without passing through registers.  Issued from inline
// assembly on purpose: the compiler then does not know that LDS is being written in the
// background and puts no vmcnt wait in front of LDS reads (as a builtin, it drains *every* copy
// in flight before any LDS transpose read, which serialises a software pipeline built on such
// copies).  The kernels wait for their copies themselves with s_waitcnt vmcnt(n) before the
// barrier that publishes a tile; the waits that the compiler adds for its own loads and stores
// can only be stricter than it thinks, never weaker, because the counter retires in order.
// The LDS address of the copy travels in m0, bound as an input operand so that the compiler
// writes the register itself and knows its value.
__device__ __forceinline__ void copy16_to_lds(rsrc_t rsrc, unsigned lds_byte_addr, int voff, int soff) {
    asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds"
                 :
                 : "v"(voff), "s"(rsrc), "s"(soff), "{m0}"(lds_byte_addr)
                 : "memory");
}
__device__ __forceinline__ void copy4_to_lds(rsrc_t rsrc, unsigned lds_byte_addr, int voff, int soff) {
    asm volatile("buffer_load_dword %0, %1, %2 offen lds"
                 :
                 : "v"(voff), "s"(rsrc), "s"(soff), "{m0}"(lds_byte_addr)
                 : "memory");
}

// ds_read_b64_tr_b16: within each group of 16 lanes, lane s supplies the address of 4
// consecutive 16-bit values D[s][0..3]; lane L receives D[4 j + L / 4][L % 4], j = 0..3: a 16 x 4
// block read row-wise comes back column-wise.
__device__ __forceinline__ s16x4_t lds_read_tr16_b64(const bf16 *p) {
    typedef s16x4_t __attribute__((address_space(3))) *lds_s16x4_ptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
}

// compile-time loop: f(std::integral_constant<int, I>) for I = 0 .. N-1
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// ---------------------------------------------------------------------------------------------
// flat-vector kernels (flat_kernels.hip)

int flat_init(photon_ctx *ctx);
void flat_free(photon_ctx *ctx);
int flat_adamw(photon_ctx *ctx, float *p, float *m, float *v, const float *g, int64_t n, int64_t t,
               float lr, const photon_adamw_hp *hp, bf16 *w16);
// AdamW over the matrices listed in a device table (flat_adamw_table), also writing the bf16 copy
// and its per-matrix transpose; the table must cover every element of the vector exactly once.
int flat_adamw_table(photon_ctx *ctx, const int64_t *offsets, const int *rows, const int *cols, int n_mats,
                     void **table_out, int *tiles_out);
int flat_adamw_tiled(photon_ctx *ctx, float *p, float *m, float *v, const float *g, int64_t n, int64_t t, float lr,
                     const photon_adamw_hp *hp, bf16 *w16, bf16 *w16t, const void *table, int n_mats, int n_tiles);
int flat_export_delta(photon_ctx *ctx, const float *global, const float *client, void *out, int dtype,
                      int64_t n);
int flat_aggregate(photon_ctx *ctx, float *global, const void *const *bufs, int K, int kind, int dtype,
                   const float *wnorm, photon_outer_opt *oo, photon_agg_metrics *metrics, int64_t n);
int flat_aggregate_static(hipStream_t st, float *global, const void *const *bufs, int K, int kind, int dtype,
                          const float *wnorm, photon_outer_opt *oo, double *norms_dev, int64_t n, int *hip_error);
int flat_client_init(photon_ctx *ctx, const float *global, float *client, float *m, float *v, int64_t n);
void fill_zero_f32(hipStream_t st, float *p, int64_t n);  // kernels_simple.hip
int flat_clip(photon_ctx *ctx, void *delta, int dtype, double max_norm, double *norm_out, int64_t n);

// ---------------------------------------------------------------------------------------------
// model (model.hip)

int model_create(photon_ctx *ctx);
void model_destroy(photon_ctx *ctx);
int model_local_steps(photon_ctx *ctx, float *params, photon_opt_state *st, const int32_t *tokens,
                      int n_steps, int n_micro, const float *lrs, const photon_adamw_hp *hp, float *loss_out);
int model_loss_grad(photon_ctx *ctx, const float *params, const int32_t *tokens, float *grads, float *loss);
