// Flash-style causal attention with in-register ALiBi bias for gfx950, bf16 operands, fp32
// softmax statistics and accumulation.  Scores s_ij = q_i . k_j / sqrt(Dh) - m_h (i - j) for
// j <= i with m_h = 2^(-8 (h+1) / H); neither the scores nor the probabilities ever reach memory.
//
// Layout trick used by all three kernels: the products are formed *transposed*
// (S^T = K Q^T, O^T = V^T P^T, ...) with v_mfma_f32_32x32x16_bf16, whose result layout gives a
// lane one column (= one query) and 16 rows (= keys).  Row-wise softmax statistics are then
// in-lane reductions plus a single exchange between the two lane halves, per-query scalars
// (running max, log-sum-exp, D_i) are per-lane scalars, and the probabilities can be fed
// straight back as the B operand of the next product: a lane half holding keys
// {4h..4h+3, 8+4h..8+4h+3} of each 16-key step is a valid k-labelling as long as the A operand
// (read from LDS with the transpose read ds_read_b64_tr_b16) uses the same one.
//
// K / V (and Q / dO in the backward kernels) tiles are copied global -> LDS directly by
// buffer_load_dwordx4 ... lds (issued from inline assembly, see copy16_to_lds), XOR-swizzled in
// 16-byte chunks, double-buffered (four stages in the dK / dV kernel).  Results whose register
// layout would give 8-byte pieces of 32 rows per store (dK, dV) leave through LDS as whole rows.

#include "kernels.h"

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// acc = 0, defined in the accumulation registers (0 * 0 + 0 through the matrix pipe).  The compiler's hazard
// recogniser does not see inside inline assembly, so the wait states it would put between the vector-ALU write
// of the operand and the MFMA reading it are spelled out.
__device__ __forceinline__ void mfma_agpr_zero(f32x16 &acc) {
    const bf16x8 z = {};
    asm volatile("s_nop 4\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %1, 0" : "=a"(acc) : "v"(z));
}

// A [ROWS][DH] bf16 tile in LDS, 16-byte chunk c of row r stored at chunk position c ^ swz(r).
// LDS serves 64 banks x 4 B = 256 B per cycle: 16 lanes of a ds_read_b128, 32 lanes of a
// ds_read_b64.  Two access patterns must both come out conflict-free:
//   rows  (frag_rows): 16 consecutive rows, the same logical chunk          -> 16 distinct slots;
//   cols  (frag_cols): rows k..k+3 (k % 4 == 0) x four consecutive chunks    -> 4 disjoint 64 B groups.
// DH = 128 (row = the 256 B bank period): swz(r) swaps the two 2-bit fields of r % 16.
// DH = 64  (two rows per bank period):    swz(r) = rotate-right of (r / 2) % 8 by one bit.
template <int DH>
struct Tile {
    static constexpr int NC = DH / 8;             // chunks per row
    static constexpr int ROWS_PER_INST = 64 / NC; // rows one 1 KiB copy instruction covers
    static __device__ __forceinline__ int swz(int r) {
        if constexpr (DH == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
        else return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
    }

    // copy rows [row0, row0 + ROWS) of a row-major matrix (row stride ld_bytes, column byte
    // offset col_bytes) into the tile; the 4 waves of the workgroup split the instructions
    template <int ROWS>
    static __device__ __forceinline__ void copy(rsrc_t rsrc, int row0, int ld_bytes, int col_bytes,
                                                bf16 *tile, int wave, int lane) {
        constexpr int NINST = ROWS / ROWS_PER_INST;
        static_assert(NINST % 4 == 0, "tile rows must split over 4 waves");
#pragma unroll
        for (int t = 0; t < NINST / 4; ++t) {
            const int inst = wave * (NINST / 4) + t;
            const int r = inst * ROWS_PER_INST + lane / NC;
            const int c = (lane % NC) ^ swz(r);
            const int voff = (lane / NC) * ld_bytes + c * 16;
            const int soff = (row0 + inst * ROWS_PER_INST) * ld_bytes + col_bytes;
            copy16_to_lds(rsrc, lds_addr(tile) + inst * 1024, voff, soff);
        }
    }

    // A/B operand with the tile's rows as the MFMA row/column index and DH as k:
    // lane -> row base + lane % 32, dh = 16 ks + 8 (lane / 32) .. + 7
    static __device__ __forceinline__ bf16x8 frag_rows(const bf16 *tile, int base, int ks, int lane) {
        const int r = base + (lane & 31);
        const int c = 2 * ks + (lane >> 5);
        return *reinterpret_cast<const bf16x8 *>(tile + r * DH + ((c ^ swz(r)) << 3));
    }

    // A operand with DH as the MFMA row index and the tile's rows as k (LDS transpose read):
    // lane -> dh = dbase + lane % 32, rows KBASE + 4 (lane / 32) + {0..3} and + 8 + {0..3}
    template <int KBASE>
    static __device__ __forceinline__ bf16x8 frag_cols(const bf16 *tile, int dbase, int lane) {
        const int g = lane >> 4, L = lane & 15;
        const int n0 = dbase + 16 * (g & 1) + 4 * (L & 3);
        const int k = 4 * (g >> 1) + (L >> 2);  // KBASE and KBASE + 8 are multiples of 8 ...
        static_assert(KBASE % 16 == 0, "the swizzle of row k must not depend on the k-step");
        // ... but swz() looks at 4 bits of the row: rows k and k + 8 differ in it, handled below
        const bf16 *a = tile + KBASE * DH + k * DH + ((((n0 >> 3) ^ swz(k)) << 3) | (n0 & 7));
        const bf16 *a8 = tile + KBASE * DH + (k + 8) * DH + ((((n0 >> 3) ^ swz(k + 8)) << 3) | (n0 & 7));
        union {
            s16x4_t h[2];
            bf16x8 v;
        } u;
        u.h[0] = lds_read_tr16_b64(a);
        u.h[1] = lds_read_tr16_b64(a8);
        return u.v;
    }

    // NR independent products acc[r] += rows(tile_r)[base_r .. base_r + 31, :] * b_r over DH:
    // the chains interleave (consecutive MFMAs never depend on each other) and the LDS fragments
    // of k-step ks + 2 are requested before the MFMAs of k-step ks are issued (three sets in flight).
    template <int NR>
    static __device__ __forceinline__ void rows_product(const bf16 *const (&tile)[NR], const int (&base)[NR],
                                                        const bf16x8 *const (&b)[NR], f32x16 (&acc)[NR], int lane) {
        constexpr int KS = DH / 16;
        bf16x8 f[3][NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) f[0][r] = frag_rows(tile[r], base[r], 0, lane);
#pragma unroll
        for (int r = 0; r < NR; ++r) f[1][r] = frag_rows(tile[r], base[r], 1, lane);
        static_for<0, KS>([&](auto ks_) {
            constexpr int ks = decltype(ks_)::value, cur = ks % 3, nn = (ks + 2) % 3;
            if constexpr (ks + 2 < KS) {
#pragma unroll
                for (int r = 0; r < NR; ++r) f[nn][r] = frag_rows(tile[r], base[r], ks + 2, lane);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < NR; ++r)
                acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[cur][r], b[r][ks], acc[r], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
    }

    // acc[i] += cols(tile)[32 i.., 16 kk..] * b(kk) over the four 16-row steps of a 64-row tile;
    // the fragments of step kk + 1 are in flight while the matrix cores run step kk.
    template <typename BF>
    static __device__ __forceinline__ void accumulate_cols(const bf16 *tile, int lane, f32x16 (&acc)[DH / 32],
                                                           BF &&bfrag) {
        constexpr int DB = DH / 32;
        bf16x8 f[2][DB];
#pragma unroll
        for (int i = 0; i < DB; ++i) f[0][i] = frag_cols<0>(tile, i * 32, lane);
        static_for<0, 4>([&](auto kk_) {
            constexpr int kk = decltype(kk_)::value;
            constexpr int cur = kk & 1, nxt = cur ^ 1;
            if constexpr (kk < 3) {
#pragma unroll
                for (int i = 0; i < DB; ++i) f[nxt][i] = frag_cols<(kk + 1) * 16>(tile, i * 32, lane);
            }
            const bf16x8 b = bfrag(kk);
#pragma unroll
            for (int i = 0; i < DB; ++i) {
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[cur][i], b, acc[i], 0, 0, 0);
            }
        });
    }
};

// Wait out the matrix pipeline after MFMAs issued from inline assembly (the compiler does not
// know about them): 3 x 8 wait states cover the 16 passes of a 32x32x16 plus its write-back.
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory"); }

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// key / row index inside a 32-block of result element e for this lane
__device__ __forceinline__ int crow(int e, int lane) { return 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3); }

// row offset of result element e that does not depend on the lane: crow(e, lane) = erow(e) + 4 (lane / 32)
__device__ __forceinline__ constexpr int erow(int e) { return 8 * (e >> 2) + (e & 3); }

// Eight consecutive result elements (one 16-key step) as a bf16 B operand.
__device__ __forceinline__ bf16x8 pack8(const f32x16 &v, int e0) {
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (bf16)v[e0 + i];
    return r;
}

// ------------------------------------------------------------------------------------ forward

constexpr int FQ = 128;  // queries per workgroup (32 per wave)
constexpr int FK = 64;   // keys per tile

template <int DH>
__global__ __launch_bounds__(256, 2) void flash_fwd_kernel(const bf16 *__restrict__ qkv, bf16 *__restrict__ o,
                                                            float *__restrict__ lse, int H, int S) {
    using T = Tile<DH>;
    constexpr int KS = DH / 16, DB = DH / 32;
    __shared__ __attribute__((aligned(1024))) bf16 smem[2 * 2 * FK * DH];  // [stage][K | V]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // 1-D grid ordered by decreasing work: all workgroups of the last (longest) query block come
    // first, so that the short ones fill the tail of the launch
    const int nqb = (S + FQ - 1) / FQ;
    const int hb = blockIdx.x % (gridDim.x / nqb);
    const int qb = nqb - 1 - blockIdx.x / (gridDim.x / nqb);
    const int hd = hb % H, b = hb / H;
    const int d = H * DH, ld = 3 * d;
    const int q0 = qb * FQ, qw = q0 + wave * 32;
    const int qi = qw + (lane & 31);  // this lane's query
    const bf16 *base = qkv + (int64_t)b * S * ld;
    const rsrc_t rs = make_rsrc(base, (uint32_t)((int64_t)S * ld * 2));

    const float slope2 = exp2f(-8.0f * (float)(hd + 1) / (float)H) * kLog2e;
    const float scale2 = rsqrtf((float)DH) * kLog2e;

    // Q^T operand: lane = query, 8 consecutive dh per k-step
    bf16x8 qf[KS];
    {
        const int qr = qi < S ? qi : S - 1;
        const bf16 *qp = base + (int64_t)qr * ld + hd * DH + 8 * (lane >> 5);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
    }

    f32x16 oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    float cb[16];  // the second 32-key block of a tile adds 32 * slope, folded into the tile offset
#pragma unroll
    for (int e = 0; e < 16; ++e) cb[e] = slope2 * (float)(crow(e, lane) - qi);

    int last = q0 + FQ - 1;
    if (last > S - 1) last = S - 1;
    const int ntiles = last / FK + 1;
    auto issue = [&](int t, int stage) {
        bf16 *ks_ = smem + stage * 2 * FK * DH;
        T::template copy<FK>(rs, t * FK, ld * 2, (d + hd * DH) * 2, ks_, wave, lane);
        T::template copy<FK>(rs, t * FK, ld * 2, (2 * d + hd * DH) * 2, ks_ + FK * DH, wave, lane);
    };
    issue(0, 0);
    for (int t = 0; t < ntiles; ++t) {
        const int stage = t & 1;
        __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();
        if (t + 1 < ntiles) issue(t + 1, stage ^ 1);
        const int j0 = t * FK;
        if (j0 > qw + 31) continue;  // every key of the tile lies after every query of this wave
        const bf16 *kt = smem + stage * 2 * FK * DH;
        const bf16 *vt = kt + FK * DH;

        f32x16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.f;
        {
            const bf16 *const tiles[2] = {kt, kt};
            const int bases[2] = {0, 32};
            const bf16x8 *const bs[2] = {qf, qf};
            T::template rows_product<2>(tiles, bases, bs, sacc, lane);
        }
        // Scores in the log2 domain, relative to the tile: s' = acc * scale + cb[e], where
        // cb[e] = slope (key offset in the tile - query) is a per-lane constant; the absolute score
        // is s' + slope * j0.  A key lies after the query exactly when cb[e] + slope * j0 > 0.
        const float tj = slope2 * (float)j0;
        const float t32 = 32.0f * slope2;
        const int thr = qi - j0 - 4 * (lane >> 5);  // key j0 + 32 kb + crow(e) > query  <=>  erow(e) > thr - 32 kb
        float mloc = -INFINITY;
        if (j0 + FK - 1 > qw) {  // diagonal tile: some keys may be after some queries
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float sc = fmaf(sacc[kb][e], scale2, cb[e]);
                    if (erow(e) > thr - 32 * kb) sc = -INFINITY;  // key after query (integer test: exact)
                    sacc[kb][e] = sc;
                    mloc = fmaxf(mloc, sc + kb * t32);
                }
        } else {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float sc = fmaf(sacc[kb][e], scale2, cb[e]);
                    sacc[kb][e] = sc;
                    mloc = fmaxf(mloc, sc + kb * t32);
                }
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
        // Lazy reference: exponents are taken relative to m_run, which only moves when the row
        // maximum has grown by more than 8 (so p <= 2^8, harmless in fp32 sums and in bf16); the
        // accumulators are rescaled only then.  The final normalisation uses the same reference,
        // so the result is the exact softmax.
        const float m_new = fmaxf(m_run, mloc + tj);
        const float m_ref = (m_new - m_run > 8.0f) ? m_new : m_run;  // first tile: m_run = -inf -> moves
        const float alpha = fast_exp2(m_run - m_ref);                // 1 when unchanged, 0 on the first tile
        m_run = m_ref;
        const float off = m_ref - tj;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float pe = fast_exp2(sacc[kb][e] - (off - kb * t32));
                sacc[kb][e] = pe;
                psum += pe;
            }
        l_run = fmaf(l_run, alpha, psum);
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int i = 0; i < DB; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[i][e] *= alpha;
        }
        // O^T += V^T P^T over the four 16-key steps of the tile
        T::accumulate_cols(vt, lane, oacc, [&](int kk) { return pack8(sacc[kk >> 1], 8 * (kk & 1)); });
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);

    l_run += __shfl_xor(l_run, 32, 64);
    if (qi < S) {
        const float inv = 1.0f / l_run;
        bf16 *op = o + ((int64_t)b * S + qi) * d + hd * DH + 4 * (lane >> 5);
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 v;
#pragma unroll
                for (int x = 0; x < 4; ++x) v[x] = (bf16)(oacc[i][4 * e4 + x] * inv);
                *reinterpret_cast<bf16x4 *>(op + i * 32 + 8 * e4) = v;
            }
        if (lane < 32) lse[((int64_t)b * H + hd) * S + qi] = m_run + __log2f(l_run);  // log2 units
    }
}

// ------------------------------------------------------------------------------------ backward
//
// With P = softmax(S), D_i = dO_i . O_i:   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - D),
// dQ = dS K / sqrt(Dh),  dK = dS^T Q / sqrt(Dh).  P is recomputed from the saved log-sum-exp.
// Two kernels, each owning its outputs (no atomics, fixed summation order): one walks the key
// tiles for a block of queries (dQ), the other walks the query tiles for a block of keys
// (dK, dV).

template <int DH>
__global__ __launch_bounds__(256, 2) void flash_bwd_dq_kernel(const bf16 *__restrict__ qkv,
                                                               const bf16 *__restrict__ o,
                                                               const bf16 *__restrict__ d_o,
                                                               const float *__restrict__ lse,
                                                               float *__restrict__ dvec, float *__restrict__ lseb,
                                                               bf16 *__restrict__ dqkv, int H, int S) {
    using T = Tile<DH>;
    constexpr int KS = DH / 16, DB = DH / 32;
    __shared__ __attribute__((aligned(1024))) bf16 smem[2 * 2 * FK * DH];  // [stage][K | V]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nqb = (S + FQ - 1) / FQ;
    const int hb = blockIdx.x % (gridDim.x / nqb);
    const int qb = nqb - 1 - blockIdx.x / (gridDim.x / nqb);  // longest first, see the forward kernel
    const int hd = hb % H, b = hb / H;
    const int d = H * DH, ld = 3 * d;
    const int q0 = qb * FQ, qw = q0 + wave * 32;
    const int qi = qw + (lane & 31);
    const int qr = qi < S ? qi : S - 1;
    const bf16 *base = qkv + (int64_t)b * S * ld;
    const rsrc_t rs = make_rsrc(base, (uint32_t)((int64_t)S * ld * 2));
    const float slope2 = exp2f(-8.0f * (float)(hd + 1) / (float)H) * kLog2e;
    const float scale = rsqrtf((float)DH), scale2 = scale * kLog2e;

    // Q^T and dO^T operands (lane = query, 8 consecutive dh per k-step); D_i = dO_i . O_i falls out of the same
    // rows: each lane sums its half of the row, the two halves meet through one exchange.  This kernel owns its
    // queries, so it also writes D_i and lse_i + slope i (log2 units: the query-dependent part of the exponent
    // p_ij = 2^(s_ij - lse_i - slope i + slope j)) for the dK / dV kernel, which runs after it.
    bf16x8 qf[KS], dof[KS];
    float Di = 0.f;
    {
        const bf16 *qp = base + (int64_t)qr * ld + hd * DH + 8 * (lane >> 5);
        const bf16 *gp = d_o + ((int64_t)b * S + qr) * d + hd * DH + 8 * (lane >> 5);
        const bf16 *op = o + ((int64_t)b * S + qr) * d + hd * DH + 8 * (lane >> 5);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
            dof[ks] = *reinterpret_cast<const bf16x8 *>(gp + 16 * ks);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 of = *reinterpret_cast<const bf16x8 *>(op + 16 * ks);
#pragma unroll
            for (int x = 0; x < 8; ++x) Di = fmaf((float)dof[ks][x], (float)of[x], Di);
        }
        Di += __shfl_xor(Di, 32, 64);
    }
    const float lse2 = lse[((int64_t)b * H + hd) * S + qr];  // saved in log2 units
    if (lane < 32 && qi < S) {
        dvec[((int64_t)b * H + hd) * S + qi] = Di;
        lseb[((int64_t)b * H + hd) * S + qi] = lse2 + slope2 * (float)qi;
    }
    // Bias of result element e relative to the 32-key block: slope (crow(e) - query) - lse, with
    // crow(e) = 8 (e / 4) + 4 (lane / 32) + e % 4.  The e % 4 part lives in four per-lane constants,
    // the 8 (e / 4) part joins the per-block offset below (same instruction count, 12 registers less).
    float cb4[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) cb4[x] = slope2 * (float)(4 * (lane >> 5) + x - qi) - lse2;

    f32x16 acc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

    int last = q0 + FQ - 1;
    if (last > S - 1) last = S - 1;
    const int ntiles = last / FK + 1;
    auto issue = [&](int t, int stage) {
        bf16 *ks_ = smem + stage * 2 * FK * DH;
        T::template copy<FK>(rs, t * FK, ld * 2, (d + hd * DH) * 2, ks_, wave, lane);
        T::template copy<FK>(rs, t * FK, ld * 2, (2 * d + hd * DH) * 2, ks_ + FK * DH, wave, lane);
    };
    issue(0, 0);
    for (int t = 0; t < ntiles; ++t) {
        const int stage = t & 1;
        __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();
        if (t + 1 < ntiles) issue(t + 1, stage ^ 1);
        const int j0 = t * FK;
        if (j0 > qw + 31) continue;
        const bf16 *kt = smem + stage * 2 * FK * DH;
        const bf16 *vt = kt + FK * DH;
        const bool diag = j0 + FK - 1 > qw;
        const float tj = slope2 * (float)j0;
        const int thr = qi - j0 - 4 * (lane >> 5);  // key after query  <=>  erow(e) > thr - 32 kb
        f32x16 sp[4];  // S^T block 0, S^T block 1, dP^T block 0, dP^T block 1; dS^T overwrites S^T
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int e = 0; e < 16; ++e) sp[r][e] = 0.f;
        {
            // two products at a time: four interleaved chains would need more fragment registers
            // than two workgroups per compute unit leave (256 per lane)
            const int bases[2] = {0, 32};
            const bf16 *const kk_[2] = {kt, kt};
            const bf16x8 *const qq_[2] = {qf, qf};
            f32x16(&s2)[2] = *reinterpret_cast<f32x16(*)[2]>(&sp[0]);
            T::template rows_product<2>(kk_, bases, qq_, s2, lane);
            const bf16 *const vv_[2] = {vt, vt};
            const bf16x8 *const gg_[2] = {dof, dof};
            f32x16(&p2)[2] = *reinterpret_cast<f32x16(*)[2]>(&sp[2]);
            T::template rows_product<2>(vv_, bases, gg_, p2, lane);
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            f32x16 &sacc = sp[kb];
            const f32x16 &pacc = sp[2 + kb];
            if (diag) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float tjk = tj + (float)(kb * 32 + 8 * (e >> 2)) * slope2;  // one per group of four
                    float pe = fast_exp2(fmaf(sacc[e], scale2, cb4[e & 3]) + tjk);
                    if (erow(e) > thr - 32 * kb) pe = 0.f;
                    sacc[e] = pe * (pacc[e] - Di);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float tjk = tj + (float)(kb * 32 + 8 * (e >> 2)) * slope2;
                    sacc[e] = fast_exp2(fmaf(sacc[e], scale2, cb4[e & 3]) + tjk) * (pacc[e] - Di);
                }
            }
        }
        T::accumulate_cols(kt, lane, acc, [&](int kk) { return pack8(sp[kk >> 1], 8 * (kk & 1)); });
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);

    if (qi < S) {
        bf16 *op = dqkv + ((int64_t)b * S + qi) * ld + hd * DH + 4 * (lane >> 5);
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 v;
#pragma unroll
                for (int x = 0; x < 4; ++x) v[x] = (bf16)(acc[i][4 * e4 + x] * scale);
                *reinterpret_cast<bf16x4 *>(op + i * 32 + 8 * e4) = v;
            }
    }
}

constexpr int BKB = 128;  // keys per workgroup (32 per wave)
constexpr int BQT = 64;   // queries per tile (two halves of 32)

// s_waitcnt immediate: vmcnt = n (low four bits and bits 15:14), the other counters left alone
constexpr int vmcnt_imm(int n) { return 0x0f70 | (n & 15) | ((n >> 4) << 14); }

// MFMAs of the pipelined loop, issued from inline assembly so that operands and accumulators stay in the register
// file this kernel assigns them (K / V operands and dK / dV in the accumulation registers, S / dP in architectural
// ones).  The compiler cannot see their hazards; none needs a wait state here: every operand written by the vector
// ALU (the bf16 packs) is a whole step old, fragments come from LDS behind a wait count, a chain's next MFMA on the
// same accumulator is at least two MFMAs away, and results are read by the vector ALU two slots (four MFMAs) or more
// after the chain's last MFMA issued (mfma_drain() where that does not hold).
__device__ __forceinline__ void mfma_v(f32x16 &acc, const bf16x8 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_v_first(f32x16 &acc, const bf16x8 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_a(f32x16 &acc, const bf16x8 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// dK / dV for a block of 128 keys, walking the query tiles at or after it.  One wave per SIMD, so
// nothing but this wave's own instruction stream can fill the matrix pipe while it does the
// element-wise work: the loop is software-pipelined over half tiles of 32 queries.  In one step a
// wave issues, interleaved slot by slot,
//   A: the MFMAs of S = Q K^T and dP = dO V^T for the half tile after the current one,
//   B: P = 2^(s - lse') and dS = P o (dP - D) for the current half tile (vector ALU),
//   C: the MFMAs of dV += dO^T P and dK += Q^T dS for the half tile before it,
// which are independent of each other inside the step.
template <int DH>
__global__ __launch_bounds__(256, 1) void flash_bwd_dkv_kernel(const bf16 *__restrict__ qkv,
                                                                const bf16 *__restrict__ d_o,
                                                                const float *__restrict__ lseb,
                                                                const float *__restrict__ dvec,
                                                                bf16 *__restrict__ dqkv, int H, int S) {
    using T = Tile<DH>;
    constexpr int KS = DH / 16, DB = DH / 32;
    constexpr int NST = 4;                    // tile stages in LDS
    constexpr int NA = 2 * KS, NC = 4 * DB;   // MFMAs of stream A and of stream C per step
    constexpr int PPS = (NA + NC) / 16;       // MFMAs per slot of a full step (16 slots = 16 result elements)
    constexpr int RING = 8, DIST = 6;         // fragment ring and prefetch distance, in MFMAs
    constexpr int TILE = BQT * DH;            // elements of one Q or dO tile
    __shared__ __attribute__((aligned(1024))) bf16 smem[NST * 2 * TILE];  // [stage][Q | dO]
    __shared__ __attribute__((aligned(256))) float stat[NST][2][BQT];     // [stage][lseb | D][query]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nkb = (S + BKB - 1) / BKB;
    const int hb = blockIdx.x % (gridDim.x / nkb);
    const int hd = hb % H, b = hb / H;
    const int d = H * DH, ld = 3 * d;
    const int jb = (blockIdx.x / (gridDim.x / nkb)) * BKB, jw = jb + wave * 32;
    const int kj = jw + (lane & 31);
    const int kr = kj < S ? kj : S - 1;
    const bf16 *base = qkv + (int64_t)b * S * ld;
    const bf16 *gbase = d_o + (int64_t)b * S * d;
    const rsrc_t rq = make_rsrc(base, (uint32_t)((int64_t)S * ld * 2));
    const rsrc_t rg = make_rsrc(gbase, (uint32_t)((int64_t)S * d * 2));
    const float slope2 = exp2f(-8.0f * (float)(hd + 1) / (float)H) * kLog2e;
    const float scale = rsqrtf((float)DH), scale2 = scale * kLog2e;
    // waves 0, 2 copy the tile's lseb, waves 1, 3 its D (the same bytes twice: every wave issues the
    // same number of copies, so one wait count serves all)
    const float *sp_ = ((wave & 1) ? dvec : lseb) + ((int64_t)b * H + hd) * S;
    const rsrc_t rs = make_rsrc(sp_, (uint32_t)(S * 4));

    // K^T and V^T operands (lane = key, 8 consecutive dh per k-step) live in the accumulation registers for the
    // whole kernel: loaded there directly, read from there by the MFMAs
    bf16x8 kf[KS], vf[KS];
    f32x16 dk[DB], dv[DB];
    const float ckj = slope2 * (float)kj;

    const int t0 = jb / BQT, t1 = S / BQT;
    // global -> LDS copies of tile t, one instruction at a time (CI = 0 .. NCP - 1: Q rows, dO rows; NCP: statistics).
    // A tile index past the last one turns every lane's offset out of range: nothing is read.
    constexpr int NCP = 2 * (BQT / T::ROWS_PER_INST / 4);
    int voffq[NCP / 2], voffg[NCP / 2];
#pragma unroll
    for (int c = 0; c < NCP / 2; ++c) {
        const int inst = wave * (NCP / 2) + c;
        const int r = inst * T::ROWS_PER_INST + lane / T::NC;
        const int cc = (lane % T::NC) ^ T::swz(r);
        voffq[c] = (lane / T::NC) * ld * 2 + cc * 16;
        voffg[c] = (lane / T::NC) * d * 2 + cc * 16;
    }
    auto copy_one = [&](auto ci_, int t, int stage) {
        constexpr int CI = decltype(ci_)::value;
        const bool valid = t < t1;
        if constexpr (CI < NCP) {
            constexpr int c = CI % (NCP / 2);
            constexpr bool G = CI >= NCP / 2;
            const int inst = wave * (NCP / 2) + c;
            bf16 *dst = smem + stage * 2 * TILE + (G ? TILE : 0);
            const int row = t * BQT + inst * T::ROWS_PER_INST;
            const int v = valid ? (G ? voffg[c] : voffq[c]) : 0x7fffffff;
            copy16_to_lds(G ? rg : rq, lds_addr(dst) + inst * 1024, v, row * (G ? d : ld) * 2 + hd * DH * 2);
        } else {
            copy4_to_lds(rs, lds_addr(&stat[stage][wave & 1][0]), valid ? lane * 4 : 0x7fffffff, t * BQT * 4);
        }
    };
    auto copy_tile = [&](int t, int stage) {
        static_for<0, NCP + 1>([&](auto ci_) { copy_one(ci_, t, stage); });
    };

    f32x16 sS[2], sP[2];       // [half] scores and dP of the half tile computed by A, consumed by B one step later
    bf16x8 pkP[2][2], pkS[2][2];  // [half][16-query step] P and dS as bf16 B operands, written by B, consumed by C
    bf16x8 fr[RING];
    f32x4 l4[2], d4[2];

    // fragment of MFMA number J of stream A (S, dP of half HALF of the tile at qt / gt) or C
    auto frag_a = [&](auto j_, auto half_, const bf16 *qt) {
        constexpr int J = decltype(j_)::value, HALF = decltype(half_)::value;
        return T::frag_rows((J & 1) ? qt + TILE : qt, 32 * HALF, J >> 1, lane);
    };
    auto frag_c = [&](auto j_, auto half_, const bf16 *qt) {
        constexpr int J = decltype(j_)::value, HALF = decltype(half_)::value;
        constexpr int kkl = J / (2 * DB), typ = (J / DB) & 1, i = J % DB;
        return T::template frag_cols<16 * (2 * HALF + kkl)>(typ ? qt : qt + TILE, i * 32, lane);
    };

    // One step.  ODD = second half of tile t.  Streams present: HA, HB, HC.  NEXT_* describe the step that
    // follows (its first DIST fragments are requested here).  Tiles: ta = tile of stream A, tb = B's, tc = C's.
    //   even step (tile t):  A half 1 of t,     B half 0 of t,  C half 1 of t - 1
    //   odd  step (tile t):  A half 0 of t + 1, B half 1 of t,  C half 0 of t;   copies of tile t + 3
    float hold_p = 0.f, hold_s = 0.f;
    auto stat_read = [&](auto g_, int stage, int half) {
        constexpr int G = decltype(g_)::value;
        const int r0 = half * 32 + 8 * (G & 3) + 4 * (lane >> 5);
        l4[G & 1] = *reinterpret_cast<const f32x4 *>(&stat[stage][0][r0]);
        d4[G & 1] = *reinterpret_cast<const f32x4 *>(&stat[stage][1][r0]);
    };
    auto step = [&](auto odd_, auto ha_, auto hb_, auto hc_, auto pre_, auto nxt_, auto mask_, int t) __attribute__((always_inline)) {
        constexpr bool ODD = decltype(odd_)::value, HA = decltype(ha_)::value, HB = decltype(hb_)::value,
                       HC = decltype(hc_)::value, PRE = decltype(pre_)::value, NXT = decltype(nxt_)::value,
                       MASK = decltype(mask_)::value;
        constexpr int HALF_A = ODD ? 0 : 1, HALF_B = ODD ? 1 : 0, HALF_C = ODD ? 0 : 1;
        constexpr int NM = (HA ? NA : 0) + (HC ? NC : 0);
        constexpr int C_FIRST = (ODD && HA) ? NC * 3 / 4 : 0;  // C MFMAs ahead of stream A in this step
        const int sa = ((ODD ? t + 1 : t) - t0) & (NST - 1), sb = (t - t0) & (NST - 1),
                  sc = ((ODD ? t : t - 1) - t0) & (NST - 1);
        const bf16 *qa = smem + sa * 2 * TILE, *qc = smem + sc * 2 * TILE;
        // position p of this step -> (is stream A, index in its stream)
        auto is_a = [](int p) constexpr { return HA && (!HC || (ODD ? (p >= C_FIRST && p < C_FIRST + NA) : p < NA)); };
        auto idx = [](int p) constexpr {
            if (!HC) return p;
            if (!HA) return p;
            if (ODD) return p < C_FIRST ? p : (p < C_FIRST + NA ? p - C_FIRST : p - NA);
            return p < NA ? p : p - NA;
        };
        auto request = [&](auto p_) {
            constexpr int P = decltype(p_)::value;
            if constexpr (P < NM) {
                if constexpr (is_a(P)) fr[P % RING] = frag_a(std::integral_constant<int, idx(P)>{}, std::integral_constant<int, HALF_A>{}, qa);
                else fr[P % RING] = frag_c(std::integral_constant<int, idx(P)>{}, std::integral_constant<int, HALF_C>{}, qc);
            } else if constexpr (NXT) {
                // the next step is the other kind with all three streams: even starts with A (half 1 of tile t + 1,
                // seen from an odd step), odd starts with C (half 0 of tile t, seen from an even step)
                constexpr int Q = P - NM;
                if constexpr (ODD) fr[P % RING] = frag_a(std::integral_constant<int, Q>{}, std::integral_constant<int, 1>{}, qa);
                else fr[P % RING] = frag_c(std::integral_constant<int, Q>{}, std::integral_constant<int, 0>{}, smem + sb * 2 * TILE);
            }
        };
        const int thr = kj - (t * BQT + 32 * HALF_B) - 4 * (lane >> 5);
        if constexpr (!PRE) static_for<0, DIST>([&](auto p_) { request(p_); });
        if constexpr (HB && !PRE) stat_read(std::integral_constant<int, 0>{}, sb, HALF_B);
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, 16>([&](auto s_) {
            constexpr int SL = decltype(s_)::value, e = SL;
            float pe = 0.f, dd = 0.f;
            // ---- vector ALU, first part: the exponential of result element SL of the current half tile
            if constexpr (HB) {
                if constexpr ((e & 3) == 0 && e + 4 < 16) stat_read(std::integral_constant<int, e / 4 + 1>{}, sb, HALF_B);
                pe = fast_exp2(fmaf(sS[HALF_B][e], scale2, ckj) - l4[(e >> 2) & 1][e & 3]);
                dd = sP[HALF_B][e] - d4[(e >> 2) & 1][e & 3];
            }
            auto mfma_at = [&](auto p_) __attribute__((always_inline)) {
                constexpr int P = decltype(p_)::value;
                if constexpr (P < NM) {
                    constexpr int J = idx(P);
                    if constexpr (is_a(P)) {
                        constexpr int ks = J >> 1;
                        if constexpr (J & 1) {
                            if constexpr (ks == 0) mfma_v_first(sP[HALF_A], fr[P % RING], vf[0]);
                            else mfma_v(sP[HALF_A], fr[P % RING], vf[ks]);
                        } else {
                            if constexpr (ks == 0) mfma_v_first(sS[HALF_A], fr[P % RING], kf[0]);
                            else mfma_v(sS[HALF_A], fr[P % RING], kf[ks]);
                        }
                    } else {
                        constexpr int kkl = J / (2 * DB), typ = (J / DB) & 1, i = J % DB;
                        if constexpr (typ) mfma_a(dk[i], fr[P % RING], pkS[HALF_C][kkl]);
                        else mfma_a(dv[i], fr[P % RING], pkP[HALF_C][kkl]);
                    }
                    request(std::integral_constant<int, P + DIST>{});
                }
            };
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (PPS == 2) {
                mfma_at(std::integral_constant<int, 2 * SL>{});
                __builtin_amdgcn_sched_barrier(0);
            }
            // ---- vector ALU, second part: mask, dS, bf16 packing; one copy instruction; next step's statistics
            if constexpr (HB) {
                if constexpr (MASK) {
                    if (erow(e) < thr) pe = 0.f;
                }
                const float ds = pe * dd;
                if constexpr (e & 1) {
                    pkP[HALF_B][e >> 3][(e & 7) - 1] = (bf16)hold_p;
                    pkP[HALF_B][e >> 3][e & 7] = (bf16)pe;
                    pkS[HALF_B][e >> 3][(e & 7) - 1] = (bf16)hold_s;
                    pkS[HALF_B][e >> 3][e & 7] = (bf16)ds;
                } else {
                    hold_p = pe;
                    hold_s = ds;
                }
                if constexpr (ODD && SL >= 1 && SL <= NCP + 1)
                    copy_one(std::integral_constant<int, SL - 1>{}, t + 3, (t + 3 - t0) & (NST - 1));
                if constexpr (NXT && SL == 12) {
                    if constexpr (ODD) stat_read(std::integral_constant<int, 4>{}, (t + 1 - t0) & (NST - 1), 0);
                    else stat_read(std::integral_constant<int, 4>{}, sb, 1);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_at(std::integral_constant<int, PPS * SL + PPS - 1>{});
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using Tt = std::true_type;
    using Ff = std::false_type;

    // The block's K and V rows come through LDS as well (whole rows, coalesced; a load straight into the operand
    // layout would touch 64 different rows per instruction): K into stage 2, V into stage 3, which the query tiles
    // do not need yet, then one 16-byte LDS read per k-step into the accumulation registers.
    {
        constexpr int NKV = BKB / T::ROWS_PER_INST / 4;  // copy instructions per wave and matrix
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int c = 0; c < NKV; ++c) {
                const int inst = wave * NKV + c;
                const int r = inst * T::ROWS_PER_INST + lane / T::NC;
                const int cc = (lane % T::NC) ^ T::swz(r);
                const int vo = jb + r < S ? (lane / T::NC) * ld * 2 + cc * 16 : 0x7fffffff;  // rows past the end: not read
                copy16_to_lds(rq, lds_addr(smem + (2 + m) * 2 * TILE) + inst * 1024, vo,
                              (jb + inst * T::ROWS_PER_INST) * ld * 2 + ((1 + m) * d + hd * DH) * 2);
            }
    }
    copy_tile(t0, 0);
    copy_tile(t0 + 1, 1);
    // (the accumulators are cleared while the copies are in flight)
#pragma unroll
    for (int i = 0; i < DB; ++i) {
        mfma_agpr_zero(dk[i]);
        mfma_agpr_zero(dv[i]);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(NCP + 1));  // K, V and tile t0 have landed, tile t0 + 1 may be in flight
    __syncthreads();
    {
        const int r = wave * 32 + (lane & 31);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const unsigned at = lds_addr(smem + 2 * 2 * TILE + r * DH + (((2 * ks + (lane >> 5)) ^ T::swz(r)) << 3));
            asm volatile("ds_read_b128 %0, %1" : "=a"(kf[ks]) : "v"(at) : "memory");
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=a"(vf[ks]) : "v"(at), "i"(2 * TILE * 2) : "memory");
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    __syncthreads();  // stages 2 and 3 are free again
    copy_tile(t0 + 2, 2);
    // prologue: A alone for half 0 of tile t0 (as the A part of an odd step of tile t0 - 1)
    step(Tt{}, Tt{}, Ff{}, Ff{}, Ff{}, Tt{}, Ff{}, t0 - 1);
    mfma_drain();  // the first step reads these results at once
    stat_read(std::integral_constant<int, 0>{}, 0, 0);
    // first tile: no half tile before it to accumulate.  Tiles t0 and t0 + 1 hold queries that precede some of
    // the block's keys (masked form); the others do not.
    step(Ff{}, Tt{}, Tt{}, Ff{}, Tt{}, Tt{}, Tt{}, t0);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(NCP + 1));  // tile t0 + 1 has landed; tile t0 + 2 may be in flight
    __syncthreads();
    step(Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, t0);
    if (t0 + 1 < t1) {
        step(Ff{}, Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, t0 + 1);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(NCP + 1));
        __syncthreads();
        step(Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, t0 + 1);
    }
    for (int t = t0 + 2; t < t1; ++t) {
        step(Ff{}, Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, Ff{}, t);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(NCP + 1));  // tile t + 1 has landed; tile t + 2 may be in flight
        __syncthreads();
        step(Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, Tt{}, Ff{}, t);
    }
    // epilogue: C alone for half 1 of the last tile
    step(Ff{}, Ff{}, Ff{}, Tt{}, Ff{}, Ff{}, Ff{}, t1);
    __builtin_amdgcn_s_waitcnt(0x0f70);
    mfma_drain();

    // Results leave through LDS: a lane holds 4 consecutive dh of one key per register group, the rows of dK and dV
    // are DH contiguous elements in memory.  Each wave stages its 32 keys x DH block (16-byte chunks XOR-swizzled by
    // the key) and writes whole rows, 16 bytes per lane.
    __syncthreads();  // every wave has finished reading the last tile
    {
        constexpr int NCH = DH / 8;        // 16-byte chunks per row
        constexpr int RPI = 64 / NCH;      // rows per store instruction
        bf16 *buf = smem + wave * (2 * 32 * DH);
        const int key = lane & 31, hh = lane >> 5;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 a, c;
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    a[x] = (bf16)(dk[i][4 * e4 + x] * scale);
                    c[x] = (bf16)dv[i][4 * e4 + x];
                }
                const int ch = ((4 * i + e4) ^ (key & (NCH - 1))) * 8 + 4 * hh;
                *reinterpret_cast<bf16x4 *>(buf + key * DH + ch) = a;
                *reinterpret_cast<bf16x4 *>(buf + 32 * DH + key * DH + ch) = c;
            }
        bf16 *gp = dqkv + ((int64_t)b * S + jw) * ld + d + hd * DH;
#pragma unroll
        for (int j = 0; j < 32 / RPI; ++j) {
            const int r = j * RPI + lane / NCH, cc = lane % NCH;
            const int at = r * DH + ((cc ^ (r & (NCH - 1))) * 8);
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(buf + at);
            const bf16x8 c = *reinterpret_cast<const bf16x8 *>(buf + 32 * DH + at);
            if (jw + r < S) {
                *reinterpret_cast<bf16x8 *>(gp + (int64_t)r * ld + cc * 8) = a;
                *reinterpret_cast<bf16x8 *>(gp + (int64_t)r * ld + d + cc * 8) = c;
            }
        }
    }
}

}  // namespace

bool attention_fwd_flash_bf16(hipStream_t st, const bf16 *qkv, bf16 *o, float *lse, int B, int H, int S, int Dh) {
    if (S % FK != 0 || (Dh != 64 && Dh != 128)) return false;
    if ((int64_t)S * 3 * H * Dh * 2 >= (int64_t)1 << 31) return false;
    const dim3 grid(((S + FQ - 1) / FQ) * H * B), block(256);
    if (Dh == 128)
        hipLaunchKernelGGL((flash_fwd_kernel<128>), grid, block, 0, st, qkv, o, lse, H, S);
    else
        hipLaunchKernelGGL((flash_fwd_kernel<64>), grid, block, 0, st, qkv, o, lse, H, S);
    return true;
}

bool attention_bwd_flash_bf16(hipStream_t st, const bf16 *qkv, const bf16 *o, const float *lse, const bf16 *d_o,
                              bf16 *dqkv, float *dvec, int B, int H, int S, int Dh) {
    if (S % FK != 0 || (Dh != 64 && Dh != 128)) return false;
    if ((int64_t)S * 3 * H * Dh * 2 >= (int64_t)1 << 31) return false;
    const dim3 gq(((S + FQ - 1) / FQ) * H * B), gk(((S + BKB - 1) / BKB) * H * B), block(256);
    float *lseb = dvec + (int64_t)B * H * S;  // second half of the scratch
    if (Dh == 128) {
        hipLaunchKernelGGL((flash_bwd_dq_kernel<128>), gq, block, 0, st, qkv, o, d_o, lse, dvec, lseb, dqkv, H, S);
        hipLaunchKernelGGL((flash_bwd_dkv_kernel<128>), gk, block, 0, st, qkv, d_o, lseb, dvec, dqkv, H, S);
    } else {
        hipLaunchKernelGGL((flash_bwd_dq_kernel<64>), gq, block, 0, st, qkv, o, d_o, lse, dvec, lseb, dqkv, H, S);
        hipLaunchKernelGGL((flash_bwd_dkv_kernel<64>), gk, block, 0, st, qkv, d_o, lseb, dvec, dqkv, H, S);
    }
    return true;
}
