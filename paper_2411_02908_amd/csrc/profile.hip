// Per-kernel-class timing with HIP events on the ctx stream: a launch of a class is bracketed by
// two events, and the pairs are summed when the profile is read.  Each pair costs a few
// microseconds of stream time, so the two classes with thousands of launches per step (GEMM,
// attention) can be sampled: every n-th launch of the class is timed, in launch order, and the
// work counted is that of the timed launches only, so that work / time stays an average rate.  Used to report
// achieved FLOP/s and bytes/s against the hardware peaks (the MFU definition of the paper's
// errata appendix: device FLOPs/s divided by the peak).

#include "common.h"

thread_local KernelTimer *g_timer = nullptr;

static size_t take_event(KernelTimer &t) {
    if (t.used == t.pool.size()) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return (size_t)-1;
        t.pool.push_back(e);
    }
    return t.used++;
}

TimedLaunch::TimedLaunch(hipStream_t stream, int cls, double work) : st(stream), rec(0), active(false) {
    KernelTimer *t = g_timer;
    if (!t || !t->on) return;
    const int64_t index = t->seen[cls]++;
    if ((cls == KC_GEMM || cls == KC_ATTN) && index % t->every != 0) return;
    const size_t e0 = take_event(*t), e1 = take_event(*t);
    if (e0 == (size_t)-1 || e1 == (size_t)-1) return;
    if (hipEventRecord(t->pool[e0], st) != hipSuccess) return;
    t->recs.push_back({cls, work, e0, e1});
    rec = t->recs.size() - 1;
    active = true;
}

TimedLaunch::~TimedLaunch() {
    if (!active) return;
    KernelTimer *t = g_timer;
    (void)hipEventRecord(t->pool[t->recs[rec].e1], st);
}

TimerScope::TimerScope(photon_ctx *ctx) { g_timer = (ctx && ctx->timer.on) ? &ctx->timer : nullptr; }
TimerScope::~TimerScope() { g_timer = nullptr; }

// Plain streaming kernels for measuring what the memory system gives: 16 bytes per lane and
// access, 2048 workgroups walking the vector in grid strides, as the flat-vector kernels do.
namespace {
typedef float probe_f4 __attribute__((ext_vector_type(4)));
constexpr int kProbeBlocks = 2048, kProbeThreads = 256;

// reads: r source arrays; writes: w destination arrays (r, w in 0..4, not both 0)
template <int R, int W>
__global__ __launch_bounds__(kProbeThreads) void stream_probe_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                                      int64_t n, float *__restrict__ sink) {
    const int64_t nvec = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kProbeThreads;
    probe_f4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x; i < nvec; i += stride) {
        probe_f4 v = {1.f, 2.f, 3.f, 4.f};
#pragma unroll
        for (int a = 0; a < R; ++a) v += *reinterpret_cast<const probe_f4 *>(src + (int64_t)a * n + 4 * i);
#pragma unroll
        for (int a = 0; a < W; ++a) *reinterpret_cast<probe_f4 *>(dst + (int64_t)a * n + 4 * i) = v;
        if (W == 0) acc += v;
    }
    if (W == 0 && acc[0] + acc[1] + acc[2] + acc[3] == 12345.678f) sink[0] = acc[0];  // keeps the reads alive
}

template <int R>
void launch_probe(int w, hipStream_t st, const float *src, float *dst, int64_t n, float *sink) {
    const dim3 g(kProbeBlocks), b(kProbeThreads);
    switch (w) {
        case 0: hipLaunchKernelGGL((stream_probe_kernel<R, 0>), g, b, 0, st, src, dst, n, sink); break;
        case 1: hipLaunchKernelGGL((stream_probe_kernel<R, 1>), g, b, 0, st, src, dst, n, sink); break;
        case 2: hipLaunchKernelGGL((stream_probe_kernel<R, 2>), g, b, 0, st, src, dst, n, sink); break;
        case 3: hipLaunchKernelGGL((stream_probe_kernel<R, 3>), g, b, 0, st, src, dst, n, sink); break;
        default: hipLaunchKernelGGL((stream_probe_kernel<R, 4>), g, b, 0, st, src, dst, n, sink); break;
    }
}
}  // namespace

extern "C" {

int photon_stream_probe(photon_ctx *ctx, int32_t reads, int32_t writes, const float *src, float *dst, int64_t n,
                        int32_t repeats, double *ms_out) {
    if (!ctx || !ms_out || reads < 0 || reads > 4 || writes < 0 || writes > 4 || reads + writes == 0) return PHOTON_EINVAL;
    if (n < 4 || n % 4 != 0 || repeats < 1 || (reads && !src) || !dst) return PHOTON_EINVAL;
    if (!aligned16(src) || !aligned16(dst)) return PHOTON_EINVAL;
    hipStream_t st = ctx->stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(ctx, hipEventCreate(&e0));
    HIP_TRY(ctx, hipEventCreate(&e1));
    float *sink = dst;  // never written when writes == 0 (the condition in the kernel does not hold)
    for (int rep = -1; rep < repeats; ++rep) {  // one untimed launch first
        if (rep == 0) (void)hipEventRecord(e0, st);
        switch (reads) {
            case 0: launch_probe<0>(writes, st, src, dst, n, sink); break;
            case 1: launch_probe<1>(writes, st, src, dst, n, sink); break;
            case 2: launch_probe<2>(writes, st, src, dst, n, sink); break;
            case 3: launch_probe<3>(writes, st, src, dst, n, sink); break;
            default: launch_probe<4>(writes, st, src, dst, n, sink); break;
        }
    }
    (void)hipEventRecord(e1, st);
    hipError_t e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    HIP_TRY(ctx, e);
    *ms_out = (double)ms / repeats;
    return PHOTON_OK;
}

int photon_profile_begin_sampled(photon_ctx *ctx, int32_t every) {
    if (!ctx || every < 1) return PHOTON_EINVAL;
    ctx->timer.on = true;
    ctx->timer.every = every;
    ctx->timer.used = 0;
    ctx->timer.recs.clear();
    for (int c = 0; c < KC_COUNT; ++c) ctx->timer.seen[c] = 0;
    return PHOTON_OK;
}

int photon_profile_begin(photon_ctx *ctx) { return photon_profile_begin_sampled(ctx, 1); }

int photon_profile_end(photon_ctx *ctx, photon_profile *out) {
    if (!ctx || !out) return PHOTON_EINVAL;
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    double ms[KC_COUNT] = {}, work[KC_COUNT] = {};
    int64_t n[KC_COUNT] = {};
    for (const KernelTimer::Rec &r : ctx->timer.recs) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, ctx->timer.pool[r.e0], ctx->timer.pool[r.e1]) != hipSuccess) continue;
        ms[r.cls] += (double)t;
        work[r.cls] += r.work;
        n[r.cls] += 1;
    }
    out->gemm_ms = ms[KC_GEMM]; out->gemm_flops = work[KC_GEMM]; out->gemm_launches = n[KC_GEMM];
    out->attn_ms = ms[KC_ATTN]; out->attn_flops = work[KC_ATTN]; out->attn_launches = n[KC_ATTN];
    out->adamw_ms = ms[KC_ADAMW]; out->adamw_bytes = work[KC_ADAMW]; out->adamw_launches = n[KC_ADAMW];
    out->agg_ms = ms[KC_AGG]; out->agg_bytes = work[KC_AGG]; out->agg_launches = n[KC_AGG];
    out->delta_ms = ms[KC_DELTA]; out->delta_bytes = work[KC_DELTA]; out->delta_launches = n[KC_DELTA];
    out->gemm_launches_total = ctx->timer.seen[KC_GEMM];
    out->attn_launches_total = ctx->timer.seen[KC_ATTN];
    ctx->timer.on = false;
    ctx->timer.recs.clear();
    ctx->timer.used = 0;
    return PHOTON_OK;
}

}  // extern "C"
