// bf16 MFMA GEMM with fp32 accumulation for gfx950 (the QKV / O / MLP projections, the tied
// LM head, and their input- and weight-gradient products).
//
// One workgroup of four wavefronts computes a 256 x 256 tile of C; each wavefront owns a
// 128 x 128 quadrant as 8 x 8 blocks of v_mfma_f32_16x16x32_bf16 (256 accumulator registers).
// The K loop advances 32 at a time; the operands are staged 64 deep: a ring of five 32 KiB LDS
// slots holds alternately a 256 x 64 tile of A and one of B, filled directly from memory by
// buffer_load_dwordx4 ... lds (no register staging).  The tiles of the next 64 and part of the
// 64 after that are in flight while the matrix cores work on the current ones, which is what it
// takes to cover the memory latency with a single wavefront per SIMD.  Operands come in two
// LDS formats, so that all three products of training read row-major tensors as they are:
//   K-contiguous  (A of NN / NT, B of NT):  tile [256 rows][64 k], fragments by ds_read_b128;
//                 a row is 128 bytes, so the copies fetch whole cache lines;
//   K-strided     (B of NN, A and B of TN): tile [64 k][256 cols], fragments by the LDS
//                 transpose read ds_read_b64_tr_b16 (two per fragment).
// Both are XOR-swizzled in 16-byte chunks on the global side of the copy so that fragment reads
// spread over the banks.  Ragged M / N edges rely on the buffer descriptor (reads past the end
// return zero) and on masked stores; K must be a multiple of 32.

#include "kernels.h"

namespace {

constexpr int BM = 256, BN = 256, BK = 32;
constexpr int NTHREADS = 256;
constexpr int BKT = 64;                // depth of a staged operand tile: two K steps
constexpr int NSLOT = 5;               // LDS ring: A(T) B(T) A(T+1) B(T+1) A(T+2) ...
constexpr int SLOT_ELEMS = BM * BKT;   // one operand tile (bf16 elements) = 32 KiB


// GELU and its derivative for the bf16 epilogues.  erf comes from the rational approximation
// 7.1.26 of Abramowitz & Stegun (absolute error < 1.5e-7, far below bf16 resolution); it shares
// its exponential exp(-x^2 / 2) with the Gaussian density of the derivative, so each value costs
// one v_exp_f32, one v_rcp_f32 and a handful of FMAs instead of a branchy libm erff.
struct GeluParts {
    float cdf;   // Phi(x) = (1 + erf(x / sqrt 2)) / 2
    float pdf;   // exp(-x^2 / 2) / sqrt(2 pi)
};
__device__ __forceinline__ GeluParts gelu_parts(float x) {
    const float ax = fabsf(x);
    const float e = __expf(-0.5f * x * x);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752440f, ax, 1.0f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float tail = 0.5f * poly * t * e;   // (1 - erf(|x| / sqrt 2)) / 2
    GeluParts r;
    r.cdf = x >= 0.f ? 1.0f - tail : tail;
    r.pdf = e * 0.39894228040143267794f;
    return r;
}
// GELU(x) = x Phi(x) and GELU'(x) = Phi(x) + x phi(x) from one evaluation
__device__ __forceinline__ void gelu_and_grad(float x, float &y, float &dy) {
    const GeluParts g = gelu_parts(x);
    y = x * g.cdf;
    dy = fmaf(x, g.pdf, g.cdf);
}

// The global side of the tile copies of one operand.  The hardware checks the per-lane offset
// register of a buffer load against the size in the descriptor and returns zero past it; the
// scalar offset takes no part in that check.  So the per-lane register carries everything that
// depends on the lane and on the copy instruction (8 registers, fixed for the whole K loop), and
// what moves with K goes into the descriptor itself: for staged tile T its base is the first
// element of the tile and its size what is left of the matrix from there -- exact to the byte
// (zero when T lies past the end of K), so no copy ever reads outside the matrix, whatever the
// tile overhang in M, N or K.
template <bool KS>
struct OperandCopy {
    int v[8];          // per-lane byte offset of copy instruction t within the tile
    uint64_t base;     // address of tile 0 of this workgroup
    int64_t left;      // bytes from there to the end of the matrix
    int64_t step;      // bytes from one staged tile to the next

    // matrix p: [rows, K] (KS = false) or [K, cols] (KS = true), leading dimension ld;
    // first = the workgroup's first row (resp. column), k_first = its first k
    __device__ __forceinline__ OperandCopy(const void *p, int rows, int cols, int ld, int first, int k_first,
                                           int lane, int wave) {
        const int64_t bytes = ((int64_t)(rows - 1) * ld + cols) * 2;
        const int64_t off0 = KS ? ((int64_t)k_first * ld + first) * 2 : ((int64_t)first * ld + k_first) * 2;
        base = reinterpret_cast<uint64_t>(p) + off0;
        left = bytes - off0;
        step = KS ? (int64_t)BKT * ld * 2 : BKT * 2;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if constexpr (!KS) {
                // one copy instruction = 8 rows x 128 B: lane -> row lane / 8, stored chunk
                // lane % 8, which holds global chunk (lane % 8) ^ ((row / 2) % 8).  Measured on
                // the chip, a ds_read_b128 of 16 rows x 16 B per lane group runs at the full
                // LDS rate with this layout (two rows fill the 256-byte bank period; the 8 rows
                // of equal parity get 8 different positions) and at half of it with 64-byte
                // rows under any swizzle tried.  Instruction t of wave w holds rows 8 (8 w + t)
                // .., so (row / 2) % 8 = 4 (t % 2) + lane / 16.
                const int swz = 4 * (t & 1) + (lane >> 4);
                const int row = 8 * (8 * wave + t) + (lane >> 3);
                v[t] = (row * ld + (((lane & 7) ^ swz) << 3)) * 2;
            } else {
                // one copy instruction = 2 k-rows x 512 B; instruction t of wave w holds rows
                // k = 8 t + 2 w + lane / 32.  Row k stores global chunk c at position
                // c ^ 4 (k % 4) ^ 2 ((k / 8) % 2).  A transpose read serves 32 lanes per cycle: two
                // groups of 16 lanes, rows (k .. k+3) and (k+8 .. k+11), 32 B of each row.  Every row
                // starts at the same bank (row pitch 512 B); the first term puts the four rows of a
                // group into four different 64-byte bank groups, the second puts the two lane groups
                // into different halves of them.
                const int k = 8 * t + 2 * wave + (lane >> 5);
                v[t] = (k * ld + (((lane & 31) ^ (4 * (k & 3)) ^ (2 * ((k >> 3) & 1))) << 3)) * 2;
            }
        }
    }
    // descriptor for staged tile T
    __device__ __forceinline__ rsrc_t tile_rsrc(int T) const {
        const int64_t adv = step * T;
        const int64_t rem = left - adv;
        return make_rsrc(reinterpret_cast<const void *>(base + adv), (uint32_t)(rem > 0 ? rem : 0));
    }
    // LDS KiB that copy instruction t of wave w fills: rows 8 kib .. (resp. k rows 2 kib, 2 kib + 1)
    static __device__ __forceinline__ int kib(int wave, int t) { return KS ? t * 4 + wave : wave * 8 + t; }
};

// One of the 8 copy instructions (1 KiB of LDS each) with which a wave fills its share of a
// staged operand tile: 16 bytes per lane from global memory straight into LDS at M0 + 16 * lane,
// without passing through registers.  Issued from inline assembly on purpose: the compiler then
// does not know that LDS is being written in the background and puts no wait for the copies in
// front of LDS reads.
// KS = false: matrix [rows, K], tile rows first.., k columns k0..k0+63  -> LDS [256][64].
// KS = true:  matrix [K, cols], tile k rows k0.., columns first..first+255 -> LDS [64][256].
template <bool KS>
__device__ __forceinline__ void load_tile_part(rsrc_t tile, const OperandCopy<KS> &oc, bf16 *lds_tile, int wave,
                                               int t) {
    asm volatile("buffer_load_dwordx4 %0, %1, 0 offen lds"
                 :
                 : "v"(oc.v[t]), "s"(tile), "{m0}"(lds_addr(lds_tile) + OperandCopy<KS>::kib(wave, t) * 1024)
                 : "memory");
}

// Per-lane LDS element offsets of the MFMA fragments (v_mfma_f32_16x16x32_bf16: a lane holds row
// or column lane % 16 and the 8 consecutive k starting at 8 (lane / 16)) inside a wave's 128-wide
// half of a staged tile, for its first K step; see read_frag for the second.
template <bool KS>
struct FragOff {
    int v[KS ? 8 : 1];
    __device__ __forceinline__ FragOff(int lane, int half /* 0 / 1: which 128 rows or columns */) {
        if constexpr (!KS) {
            // row lane % 16, k chunk lane / 16; 16-row block i adds i * 16 * BKT (the swizzle term
            // (row / 2) % 8 does not change with i)
            const int row = half * 128 + (lane & 15);
            v[0] = row * BKT + ((((lane >> 4) ^ ((row >> 1) & 7))) << 3);
        } else {
            // v[j]: 16-column block j.  Lane group g = lane / 16 reads k rows 8 g + L / 4 (and 4
            // rows further for the second half) x 16 columns, 4 per lane; the transpose hands lane
            // L column L with 4 consecutive k.
            const int g = lane >> 4, L = lane & 15;
            const int k = 8 * g + (L >> 2);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int n0 = half * 128 + j * 16 + 4 * (L & 3);
                v[j] = k * BN + ((((n0 >> 3) ^ (4 * (k & 3)) ^ (2 * (g & 1))) << 3) | (n0 & 7));
            }
        }
    }
};

// Fragment of 16-block `blk` for K step `s` (0 / 1) of a staged tile: all 32 k of that step.
// K-strided tiles are read with the LDS transpose read (ds_read_b64_tr_b16: within 16 lanes, a
// 16 x 4 block read row-wise comes back column-wise).
template <bool KS>
__device__ __forceinline__ bf16x8 read_frag(const bf16 *lds_tile, const FragOff<KS> &fo, int blk, int s) {
    if constexpr (!KS) {
        // the second step's chunks are 4 .. 7: the swizzled position differs in bit 2
        return *reinterpret_cast<const bf16x8 *>(lds_tile + (fo.v[0] ^ (s * 32)) + blk * 16 * BKT);
    } else {
        const bf16 *p = lds_tile + fo.v[blk] + s * 32 * BN;
        union {
            s16x4_t h[2];
            bf16x8 v;
        } u;
        u.h[0] = lds_read_tr16_b64(p);
        u.h[1] = lds_read_tr16_b64(p + 4 * BN);
        return u.v;
    }
}

// acc += a b on the 16x16x32 matrix instruction, with the accumulator pinned to the accumulation
// registers.  Written as assembly because the compiler, given the builtin and 64 four-register
// accumulators, keeps half of them in ordinary registers and copies them across in every K step
// (hundreds of moves per step).  The operands come straight from LDS reads (the compiler waits
// for those before any use, assembly included); an accumulator is only ever read by the same
// instruction form, which the hardware interlocks, until mfma_drain() after the K loop.
__device__ __forceinline__ void mfma_acc(f32x4 &acc, const bf16x8 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// The wait states between the last matrix instruction and an ordinary read of its result, which
// the compiler cannot place for instructions it does not see.
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

constexpr int EPI_PARTIAL = 5;  // split-K: raw fp32 partial tile to the workspace, epilogue deferred

// PAIR: one launch computes two independent products of the same operand form and epilogue;
// workgroups [0, tiles_m * tiles_n) belong to the first, the rest to the second.
template <bool AKS, bool BKS, int EPI, bool PAIR = false>
__global__ __launch_bounds__(NTHREADS, 1) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n,
                                                                float *__restrict__ partial, GemmArgs g2 = GemmArgs(),
                                                                int tiles_m2 = 0, int tiles_n2 = 0) {
    // ring of operand tiles: slot (2 T) % 5 holds A's tile T, slot (2 T + 1) % 5 B's
    __shared__ __attribute__((aligned(1024))) bf16 smem[NSLOT * SLOT_ELEMS];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // tile order: consecutive workgroup ids go to different XCDs (round-robin over 8), so give
    // each XCD a contiguous range of tiles, walked in column-major groups of 8 tile rows to
    // keep its L2 working set small.
    int bid = blockIdx.x;
    if constexpr (PAIR) {
        if (bid >= tiles_m * tiles_n) {  // uniform over the workgroup
            bid -= tiles_m * tiles_n;
            g = g2;
            tiles_m = tiles_m2;
            tiles_n = tiles_n2;
        }
    }
    const int ntiles = tiles_m * tiles_n;
    {
        const int per = ntiles >> 3;
        if (bid < per * 8) bid = (bid & 7) * per + (bid >> 3);
    }
    constexpr int GROUP = 8;
    const int in_group = GROUP * tiles_n;
    const int gid = bid / in_group;
    const int first_m = gid * GROUP;
    const int gsize = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
    const int tm = first_m + (bid % in_group) % gsize;
    const int tn = (bid % in_group) / gsize;
    const int m0 = tm * BM, n0 = tn * BN;

    const FragOff<AKS> fa(lane, wm);
    const FragOff<BKS> fb(lane, wn);

    // 16 x 16 blocks of the wave's 128 x 128.  The MFMAs take B's fragment as their first operand
    // and A's as the second, i.e. they compute the transposed block: a lane then holds four
    // consecutive columns 16 j + 4 (lane / 16) + e of row 16 i + lane % 16, which the epilogue can
    // move 16 bytes at a time.
    f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // this workgroup's share of the K loop (gridDim.y > 1: split-K)
    const int nk_all = g.K / BK;
    const int kt_begin = (int)((int64_t)nk_all * blockIdx.y / gridDim.y);
    const int nk = (int)((int64_t)nk_all * (blockIdx.y + 1) / gridDim.y) - kt_begin;
    // A is [M, K] (or [K, M] for TN), B is [K, N] (or [N, K] for NT)
    const OperandCopy<AKS> oa(g.A, AKS ? g.K : g.M, AKS ? g.M : g.K, g.lda, m0, kt_begin * BK, lane, wave);
    const OperandCopy<BKS> ob(g.B, BKS ? g.K : g.N, BKS ? g.N : g.K, g.ldb, n0, kt_begin * BK, lane, wave);
    // copy instruction t (0..7) of this wave's share of a staged tile of A (resp. B), described
    // by `tile`, into `slot`
    auto issue_a = [&](rsrc_t tile, int slot, int t) {
        load_tile_part<AKS>(tile, oa, smem + slot * SLOT_ELEMS, wave, t);
    };
    auto issue_b = [&](rsrc_t tile, int slot, int t) {
        load_tile_part<BKS>(tile, ob, smem + slot * SLOT_ELEMS, wave, t);
    };

    // The matrix instruction is the 16x16x32 one: with random-mantissa operands the chip sustains
    // about 2.0 PFLOP/s of it under its power limit, against 1.4 - 1.65 of the 32x32x16 form
    // (registers only, no memory), so it is the shape that a power-bound GEMM wants.  A K step
    // is one k = 32 slab: 8 A and 8 B fragments, 64 MFMAs, in two halves of 32 (A blocks 0..3,
    // then 4..7).  Fragments run ahead of the MFMAs in registers: A blocks 4..7 of this step are
    // read during its first half, A blocks 0..3 and all of B of the next step during its second
    // half.
    // A trip of the loop is the two K steps of staged tiles A(T), B(T).  In its first step the
    // copies of A(T+2) go out, one per group of eight MFMAs, into the slot that B(T-1) left; in
    // the second half of its second step those of B(T+2), two per group, into the slot of A(T).
    // The only barrier of the trip sits in the middle of the second step: before it a wave waits
    // until its own copies of A(T+1) and B(T+1) have landed (the 8 copies of A(T+2) may still be
    // in flight) and until its last fragment reads of A(T) are complete; after it every wave's
    // part of the next tiles is visible and the slots of A(T), B(T) are free.  A copy is issued
    // at least 1.5 K steps before the wait that needs it.
    // With one wave per SIMD nothing else fills the matrix pipe while this wave issues other
    // instructions, and the pipe takes a new MFMA every 16 cycles -- four issue slots.  So the
    // LDS reads and copy instructions are dealt out one at a time between consecutive MFMAs
    // (a scheduling fence after every MFMA keeps them there); issued in bunches they cost the
    // pipe a third of its time.
    // Copies for tiles past the end of K are issued all the same, so that the count of
    // outstanding copies stays fixed: the range check of their descriptor turns them into zeros,
    // and they land in slots that are not read any more.
#pragma unroll
    for (int t = 0; t < 8; ++t) issue_a(oa.tile_rsrc(0), 0, t);
#pragma unroll
    for (int t = 0; t < 8; ++t) issue_b(ob.tile_rsrc(0), 1, t);
#pragma unroll
    for (int t = 0; t < 8; ++t) issue_a(oa.tile_rsrc(1), 2, t);
#pragma unroll
    for (int t = 0; t < 8; ++t) issue_b(ob.tile_rsrc(1), 3, t);
    bf16x8 a_lo[2][4], a_hi[4], bfr[2][8];
    __builtin_amdgcn_s_waitcnt(0x4f70);  // vmcnt(16): A(0), B(0)
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int j = 0; j < 8; ++j) bfr[0][j] = read_frag<BKS>(smem + SLOT_ELEMS, fb, j, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) a_lo[0][i] = read_frag<AKS>(smem, fa, i, 0);

    int T = 0;
    int slot_a = 0, slot_b = 1;  // of A(T), B(T)
    // K step u (0 / 1) of the trip, reading fragment buffers u and filling u ^ 1
    auto k_step = [&](auto u_) {
        constexpr int u = decltype(u_)::value;
        const int slot_a_next = slot_a + 2 >= NSLOT ? slot_a + 2 - NSLOT : slot_a + 2;
        const int slot_b_next = slot_b + 2 >= NSLOT ? slot_b + 2 - NSLOT : slot_b + 2;
        const int slot_b_prev = slot_b + 3 >= NSLOT ? slot_b + 3 - NSLOT : slot_b + 3;
        const bf16 *as = smem + slot_a * SLOT_ELEMS;
        // the next step's tiles: the same ones (second step), or A(T+1), B(T+1)
        const bf16 *as_next = smem + (u == 0 ? slot_a : slot_a_next) * SLOT_ELEMS;
        const bf16 *bs_next = smem + (u == 0 ? slot_b : slot_b_next) * SLOT_ELEMS;
        const rsrc_t tile_next = u == 0 ? oa.tile_rsrc(T + 2) : ob.tile_rsrc(T + 2);  // copied in this step
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                mfma_acc(acc[i][j], bfr[u][j], a_lo[u][i]);
                if (u == 0 && j == 1) issue_a(tile_next, slot_b_prev, i);
                // A blocks 4..7 of this step: all requested by the middle of group 2, so that
                // the wait ahead of the barrier finds them done
                if (i == 0 && j == 3) a_hi[0] = read_frag<AKS>(as, fa, 4, u);
                if (i == 0 && j == 6) a_hi[1] = read_frag<AKS>(as, fa, 5, u);
                if (i == 1 && j == 3) a_hi[2] = read_frag<AKS>(as, fa, 6, u);
                if (i == 2 && j == 3) a_hi[3] = read_frag<AKS>(as, fa, 7, u);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if constexpr (u == 1) {
            // vmcnt(8): this wave's copies of A(T+1), B(T+1) have landed; lgkmcnt(0): its
            // fragment reads of A(T) are complete, so that after the barrier the slot may be refilled
            __builtin_amdgcn_s_waitcnt(0x0078);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                mfma_acc(acc[4 + i][j], bfr[u][j], a_hi[i]);
                if (u == 0 && j == 1) issue_a(tile_next, slot_b_prev, 4 + i);
                if (u == 1 && j == 1) issue_b(tile_next, slot_a, 2 * i);
                if (u == 1 && j == 5) issue_b(tile_next, slot_a, 2 * i + 1);
                // the next step's fragments in the order it needs them, over the first three
                // groups
                if (i < 3 && (j & 1) == 0) {
                    constexpr int order[12] = {8, 0, 1, 2, 3, 4, 5, 6, 7, 9, 10, 11};  // 0..7: B block, 8..11: A block
                    const int f = order[4 * i + j / 2];
                    if (f < 8)
                        bfr[u ^ 1][f] = read_frag<BKS>(bs_next, fb, f, u ^ 1);
                    else
                        a_lo[u ^ 1][f - 8] = read_frag<AKS>(as_next, fa, f - 8, u ^ 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if constexpr (u == 1) {
            ++T;
            slot_a = slot_a_next;
            slot_b = slot_b_next;
        }
    };
    // two K steps per trip
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        k_step(std::integral_constant<int, 0>());
        k_step(std::integral_constant<int, 1>());
    }
    if (kt < nk) k_step(std::integral_constant<int, 0>());  // odd number of K steps
    __builtin_amdgcn_s_waitcnt(0x0f70);
    mfma_drain();

    // Epilogue.  A lane holds four consecutive columns of one row of each 16 x 16 block, 16 rows
    // per lane group: stored as they are, each row would get 32-byte pieces.  Each wave therefore
    // passes its quadrant through LDS, 32 rows x 128 columns at a time, and comes back with 8
    // consecutive columns of one row per lane: all global traffic of the epilogue (C, residual R,
    // pre-activation H) is then 16-byte (bf16) or 2 x 16-byte (fp32) per lane and contiguous
    // over 16 lanes.
    __syncthreads();  // every wave has finished reading the operand tiles (the staging area reuses them)
    constexpr int EP_LD = 132;  // floats per staged row: 16 rows x 4 lane groups spread evenly over the banks
    float *stage = reinterpret_cast<float *>(smem) + wave * (32 * EP_LD);
    const bool vec_ok = (g.ldc % 8 == 0) && (g.N % 8 == 0);
    // What an epilogue reads from memory (saved GELU', the residual, or the gradient being
    // accumulated into) is requested for a whole pass before the pass's tile goes through LDS, so
    // that the memory latency runs under the staging instead of once per row.
    constexpr bool PRE_H = EPI == EPI_DGELU, PRE_F = EPI == EPI_RESID || EPI == EPI_ACCUM;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bf16x8 pre_h[PRE_H ? 8 : 1];
        f32x4 pre_f[PRE_F ? 8 : 1][2];
        if constexpr (PRE_H || PRE_F) {
            const bool want = vec_ok && (EPI != EPI_ACCUM || g.beta != 0.f);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int q = lane + 64 * t;
                const int row = m0 + wm * 128 + i * 32 + (q >> 4);
                const int col = n0 + wn * 128 + ((q & 15) << 3);
                const int64_t idx = (int64_t)row * g.ldc + col;
                const bool in = want && row < g.M && col < g.N;
                if constexpr (PRE_H) {
                    pre_h[t] = bf16x8{};
                    if (in) pre_h[t] = *reinterpret_cast<const bf16x8 *>(reinterpret_cast<const bf16 *>(g.H) + idx);
                } else {
                    const float *src = EPI == EPI_RESID ? g.R : reinterpret_cast<const float *>(g.C);
                    pre_f[t][0] = pre_f[t][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (in) {
                        pre_f[t][0] = *reinterpret_cast<const f32x4 *>(src + idx);
                        pre_f[t][1] = *reinterpret_cast<const f32x4 *>(src + idx + 4);
                    }
                }
            }
        }
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                *reinterpret_cast<f32x4 *>(stage + (16 * h + (lane & 15)) * EP_LD + j * 16 + 4 * (lane >> 4)) =
                    acc[2 * i + h][j];
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int q = lane + 64 * t;
            const int r = q >> 4, c8 = (q & 15) << 3;
            const int row = m0 + wm * 128 + i * 32 + r;
            const int col = n0 + wn * 128 + c8;
            float v[8];
            {
                const f32x4 lo = *reinterpret_cast<const f32x4 *>(stage + r * EP_LD + c8);
                const f32x4 hi = *reinterpret_cast<const f32x4 *>(stage + r * EP_LD + c8 + 4);
#pragma unroll
                for (int x = 0; x < 4; ++x) { v[x] = lo[x]; v[x + 4] = hi[x]; }
            }
            if (row >= g.M || col >= g.N) continue;
            if constexpr (EPI == EPI_PARTIAL) {
                float *pp = partial + ((int64_t)blockIdx.y * g.M + row) * g.N + col;
                if (g.N % 8 == 0) {
                    *reinterpret_cast<f32x4 *>(pp) = f32x4{v[0], v[1], v[2], v[3]};
                    *reinterpret_cast<f32x4 *>(pp + 4) = f32x4{v[4], v[5], v[6], v[7]};
                } else {
                    for (int x = 0; x < 8 && col + x < g.N; ++x) pp[x] = v[x];
                }
                continue;
            }
            const int64_t idx = (int64_t)row * g.ldc + col;
            if (vec_ok) {
                if constexpr (EPI == EPI_STORE) {
                    bf16x8 o;
#pragma unroll
                    for (int x = 0; x < 8; ++x) o[x] = (bf16)v[x];
                    *reinterpret_cast<bf16x8 *>(reinterpret_cast<bf16 *>(g.C) + idx) = o;
                } else if constexpr (EPI == EPI_RESID) {
                    const f32x4 r0 = pre_f[t][0], r1 = pre_f[t][1];
                    float *cp = reinterpret_cast<float *>(g.C) + idx;
                    *reinterpret_cast<f32x4 *>(cp) = f32x4{r0[0] + v[0], r0[1] + v[1], r0[2] + v[2], r0[3] + v[3]};
                    *reinterpret_cast<f32x4 *>(cp + 4) = f32x4{r1[0] + v[4], r1[1] + v[5], r1[2] + v[6], r1[3] + v[7]};
                } else if constexpr (EPI == EPI_GELU) {
                    bf16x8 dg, u;
#pragma unroll
                    for (int x = 0; x < 8; ++x) {
                        float y, dy;
                        gelu_and_grad(v[x], y, dy);
                        u[x] = (bf16)y;
                        dg[x] = (bf16)dy;
                    }
                    *reinterpret_cast<bf16x8 *>(reinterpret_cast<bf16 *>(g.C) + idx) = dg;
                    *reinterpret_cast<bf16x8 *>(reinterpret_cast<bf16 *>(g.C2) + idx) = u;
                } else if constexpr (EPI == EPI_DGELU) {
                    const bf16x8 h = pre_h[t];
                    bf16x8 o;
#pragma unroll
                    for (int x = 0; x < 8; ++x) o[x] = (bf16)(v[x] * (float)h[x]);
                    *reinterpret_cast<bf16x8 *>(reinterpret_cast<bf16 *>(g.C) + idx) = o;
                } else {
                    float *cp = reinterpret_cast<float *>(g.C) + idx;
                    const f32x4 c0 = pre_f[t][0] * g.beta, c1 = pre_f[t][1] * g.beta;  // zeros when beta == 0
                    *reinterpret_cast<f32x4 *>(cp) = f32x4{c0[0] + v[0], c0[1] + v[1], c0[2] + v[2], c0[3] + v[3]};
                    *reinterpret_cast<f32x4 *>(cp + 4) = f32x4{c1[0] + v[4], c1[1] + v[5], c1[2] + v[6], c1[3] + v[7]};
                }
            } else {
                for (int x = 0; x < 8 && col + x < g.N; ++x) {
                    const float val = v[x];
                    if constexpr (EPI == EPI_STORE) {
                        reinterpret_cast<bf16 *>(g.C)[idx + x] = (bf16)val;
                    } else if constexpr (EPI == EPI_RESID) {
                        reinterpret_cast<float *>(g.C)[idx + x] = g.R[idx + x] + val;
                    } else if constexpr (EPI == EPI_GELU) {
                        float y, dy;
                        gelu_and_grad(val, y, dy);
                        reinterpret_cast<bf16 *>(g.C)[idx + x] = (bf16)dy;
                        reinterpret_cast<bf16 *>(g.C2)[idx + x] = (bf16)y;
                    } else if constexpr (EPI == EPI_DGELU) {
                        reinterpret_cast<bf16 *>(g.C)[idx + x] =
                            (bf16)(val * (float)reinterpret_cast<const bf16 *>(g.H)[idx + x]);
                    } else {
                        float *c = reinterpret_cast<float *>(g.C) + idx + x;
                        *c = (g.beta != 0.f ? g.beta * *c : 0.f) + val;
                    }
                }
            }
        }
        __syncthreads();
    }
}

// Sum of the split-K partial tiles in split order, then the epilogue.  Four columns per thread.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmArgs g, const float *__restrict__ partial, int splits) {
    const int64_t quads = (int64_t)g.M * (g.N / 4);
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= quads) return;
    const int row = (int)(q / (g.N / 4)), col = (int)(q % (g.N / 4)) * 4;
    f32x4 s = *reinterpret_cast<const f32x4 *>(partial + (int64_t)row * g.N + col);
    for (int p = 1; p < splits; ++p)
        s += *reinterpret_cast<const f32x4 *>(partial + ((int64_t)p * g.M + row) * g.N + col);
    const int64_t idx = (int64_t)row * g.ldc + col;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const float v = s[x];
        if constexpr (EPI == EPI_STORE) {
            reinterpret_cast<bf16 *>(g.C)[idx + x] = (bf16)v;
        } else if constexpr (EPI == EPI_RESID) {
            reinterpret_cast<float *>(g.C)[idx + x] = g.R[idx + x] + v;
        } else if constexpr (EPI == EPI_GELU) {
            float y, dy;
            gelu_and_grad(v, y, dy);
            reinterpret_cast<bf16 *>(g.C)[idx + x] = (bf16)dy;
            reinterpret_cast<bf16 *>(g.C2)[idx + x] = (bf16)y;
        } else if constexpr (EPI == EPI_DGELU) {
            reinterpret_cast<bf16 *>(g.C)[idx + x] = (bf16)(v * (float)reinterpret_cast<const bf16 *>(g.H)[idx + x]);
        } else {
            float *c = reinterpret_cast<float *>(g.C) + idx + x;
            *c = (g.beta != 0.f ? g.beta * *c : 0.f) + v;
        }
    }
}

// set by the calling thread for the ctx it is running (distinct ctxs may run on distinct threads)
thread_local float *g_splitk_ws = nullptr;
thread_local size_t g_splitk_bytes = 0;

template <bool AKS, bool BKS>
void launch_epi(hipStream_t st, GemmEpi epi, const GemmArgs &g) {
    const int tm = (g.M + BM - 1) / BM, tn = (g.N + BN - 1) / BN;
    const int tiles = tm * tn, nk = g.K / BK;
    const dim3 block(NTHREADS);
    // Few tiles and a long K loop: split K over several workgroups per tile so that the whole
    // chip works, partial sums going through a float32 workspace (fixed order, no atomics).
    int splits = 1;
    if (tiles <= 128 && g.N % 4 == 0) {
        splits = 256 / tiles;
        if (splits > 8) splits = 8;
        while (splits > 1 && (nk / splits < 16 || (size_t)splits * g.M * g.N * sizeof(float) > g_splitk_bytes)) --splits;
    }
    if (splits > 1) {
        hipLaunchKernelGGL((gemm_mfma_kernel<AKS, BKS, EPI_PARTIAL>), dim3(tiles, splits), block, 0, st, g, tm, tn,
                           g_splitk_ws);
        const dim3 rgrid((unsigned)(((int64_t)g.M * (g.N / 4) + 255) / 256));
        switch (epi) {
            case EPI_STORE: hipLaunchKernelGGL((splitk_reduce_kernel<EPI_STORE>), rgrid, dim3(256), 0, st, g, g_splitk_ws, splits); break;
            case EPI_RESID: hipLaunchKernelGGL((splitk_reduce_kernel<EPI_RESID>), rgrid, dim3(256), 0, st, g, g_splitk_ws, splits); break;
            case EPI_GELU: hipLaunchKernelGGL((splitk_reduce_kernel<EPI_GELU>), rgrid, dim3(256), 0, st, g, g_splitk_ws, splits); break;
            case EPI_DGELU: hipLaunchKernelGGL((splitk_reduce_kernel<EPI_DGELU>), rgrid, dim3(256), 0, st, g, g_splitk_ws, splits); break;
            default: hipLaunchKernelGGL((splitk_reduce_kernel<EPI_ACCUM>), rgrid, dim3(256), 0, st, g, g_splitk_ws, splits); break;
        }
        return;
    }
    const dim3 grid(tiles);
    float *none = nullptr;
    switch (epi) {
        case EPI_STORE: hipLaunchKernelGGL((gemm_mfma_kernel<AKS, BKS, EPI_STORE>), grid, block, 0, st, g, tm, tn, none); break;
        case EPI_RESID: hipLaunchKernelGGL((gemm_mfma_kernel<AKS, BKS, EPI_RESID>), grid, block, 0, st, g, tm, tn, none); break;
        case EPI_GELU: hipLaunchKernelGGL((gemm_mfma_kernel<AKS, BKS, EPI_GELU>), grid, block, 0, st, g, tm, tn, none); break;
        case EPI_DGELU: hipLaunchKernelGGL((gemm_mfma_kernel<AKS, BKS, EPI_DGELU>), grid, block, 0, st, g, tm, tn, none); break;
        default: hipLaunchKernelGGL((gemm_mfma_kernel<AKS, BKS, EPI_ACCUM>), grid, block, 0, st, g, tm, tn, none); break;
    }
}

}  // namespace

void gemm_set_splitk_workspace(float *ws, size_t bytes) {
    g_splitk_ws = ws;
    g_splitk_bytes = bytes;
}

// What the tile kernel handles; the rest goes to the plain kernel.
static bool covered(GemmOp op, const GemmArgs &g) {
    if (g.K < BK || g.K % BK != 0) return false;
    if (g.M < 1 || g.N < 8) return false;
    // 16-byte global chunks: leading dimensions and the clamped edges must be multiples of 8
    if (g.lda % 8 != 0 || g.ldb % 8 != 0) return false;
    if ((reinterpret_cast<uintptr_t>(g.A) | reinterpret_cast<uintptr_t>(g.B)) & 15u) return false;
    if ((reinterpret_cast<uintptr_t>(g.C) | reinterpret_cast<uintptr_t>(g.C2) | reinterpret_cast<uintptr_t>(g.R) |
         reinterpret_cast<uintptr_t>(g.H)) & 15u)
        return false;  // the epilogue moves 16-byte vectors
    if (op == GEMM_TN && (g.M % 8 != 0 || g.M < 8)) return false;
    if (op != GEMM_NT && g.N % 8 != 0) return false;
    // operand byte offsets are 32-bit (buffer addressing), with a tile of slack past the end
    const int64_t rows_a = op == GEMM_TN ? g.K : g.M, rows_b = op == GEMM_NT ? g.N : g.K;
    if ((rows_a + 512) * g.lda * 2 >= ((int64_t)1 << 31) || (rows_b + 512) * g.ldb * 2 >= ((int64_t)1 << 31)) return false;
    return (int64_t)g.M * g.N >= 128 * 128;  // tiny problems are not worth a 256 x 256 tile
}

// Two weight-gradient products (TN, fp32 accumulate) in one launch when their tiles together fit
// one wave of workgroups (one per compute unit): the smaller one then rides along in compute
// units that the larger one would leave idle, instead of a launch of its own with split K.
bool gemm_mfma_bf16_pair_covered(const GemmArgs &g1, const GemmArgs &g2) {
    if (g1.K != g2.K || !covered(GEMM_TN, g1) || !covered(GEMM_TN, g2)) return false;
    const int t1 = ((g1.M + BM - 1) / BM) * ((g1.N + BN - 1) / BN);
    const int t2 = ((g2.M + BM - 1) / BM) * ((g2.N + BN - 1) / BN);
    return t1 + t2 <= 256 && t1 % 8 == 0;  // t1 % 8: the second product's tiles keep their XCD mapping
}

bool gemm_mfma_bf16_pair_tn_accum(hipStream_t st, const GemmArgs &g1, const GemmArgs &g2) {
    if (!gemm_mfma_bf16_pair_covered(g1, g2)) return false;
    const int tm1 = (g1.M + BM - 1) / BM, tn1 = (g1.N + BN - 1) / BN;
    const int tm2 = (g2.M + BM - 1) / BM, tn2 = (g2.N + BN - 1) / BN;
    const int t1 = tm1 * tn1, t2 = tm2 * tn2;
    float *none = nullptr;
    hipLaunchKernelGGL((gemm_mfma_kernel<true, true, EPI_ACCUM, true>), dim3(t1 + t2), dim3(NTHREADS), 0, st, g1, tm1,
                       tn1, none, g2, tm2, tn2);
    return true;
}

bool gemm_mfma_bf16(hipStream_t st, GemmOp op, GemmEpi epi, const GemmArgs &g) {
    if (!covered(op, g)) return false;
    switch (op) {
        case GEMM_NN: launch_epi<false, true>(st, epi, g); break;
        case GEMM_NT: launch_epi<false, false>(st, epi, g); break;
        default: launch_epi<true, true>(st, epi, g); break;
    }
    return true;
}
