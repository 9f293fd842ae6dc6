// bf16 x bf16 -> fp32 GEMM, C = alpha A B^T, on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Both operands are K-contiguous ("NT"): every contraction of the Hessian build is arranged that way (activations
// are kept in a transposed copy where the token axis is the contraction axis), so one kernel shape serves X^T X,
// the projections, Q K^T, A X and the dominant Y^T Y.
//
// Two kernels share the 256 x 256 output tile per workgroup, the MFMA shape and the launch order of the tiles:
//   gemm_bf16_nt_fast_kernel  (K a multiple of 32: every launch of the Hessian build and of the grid search) copies global
//                             memory straight into a ring of LDS stages and runs 8 wavefronts; described at its definition;
//   gemm_bf16_nt_kernel       (any K that is a multiple of 8) stages through registers: 4 wavefronts (2 x 2), each owning
//                             128 x 128 as 4 x 4 MFMA tiles of 32 x 32 (256 fp32 accumulators per lane), 64-deep k-steps,
//                             two LDS stages, one barrier per k-step.
// LDS rows of the register-staged kernel are 128 bytes (64 bf16); the LDS has 64 banks (256 bytes), so two consecutive rows
// fill one bank line and a 128-bit access is served 16 lanes at a time: the 16-byte chunks of a row are XOR-swizzled with
// (row / 2) % 8, which makes the 16 rows read by 16 consecutive lanes (and the two rows written by them) hit 16 different
// bank groups (measured: SQ_LDS_BANK_CONFLICT = 0).
// The tiles of a launch are handed out so that the 32 CUs of an XCD (workgroups are dealt to the eight XCDs round-robin)
// work on a compact block of ONE batch entry and share operand panels through that XCD's L2: see work_item / tile_order.
#include "internal.h"
#include <stdlib.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BM = 256, BN = 256, BK = 64;

struct Args {
    int M, N, K;
    float alpha;
    const __hip_bfloat16* A; long long lda;
    const __hip_bfloat16* B; long long ldb;
    void* C; long long ldc;
    int c_bf16, accumulate, flags;
    int batch_inner, kseg;
    long long sA1, sA2, sB1, sB2, sC1, sC2;
    const int* tile_order;      // (tm << 16 | tn) of the tiles of one batch entry, in launch order
    int ntiles;                 // tiles per batch entry
    long long nitems, per;      // batch * ntiles work items; per = items per XCD
};

// Work item of this workgroup.  Workgroups are dealt to the eight XCDs round-robin by their linear number, so workgroup
// w runs on XCD w % 8.  XCD x takes the contiguous run [x * per, (x + 1) * per) of the item list, which is batch-major:
// with a batch of 8 or more an XCD works through whole batch entries one after the other, its 32 CUs on 32 consecutive
// tiles of the host-built order (a compact block of the output sharing few operand panels through that XCD's L2).
__device__ __forceinline__ bool work_item(const Args& g, int& z, int& tm, int& tn) {
    const long long loc = blockIdx.x >> 3;
    const long long item = (long long)(blockIdx.x & 7) * g.per + loc;
    if (loc >= g.per || item >= g.nitems) return false;
    z = (int)(item / g.ntiles);
    const int packed = g.tile_order[(int)(item - (long long)z * g.ntiles)];
    tm = __builtin_amdgcn_readfirstlane(packed >> 16); tn = __builtin_amdgcn_readfirstlane(packed & 0xffff);
    z = __builtin_amdgcn_readfirstlane(z);
    return true;
}

__device__ __forceinline__ void load_tile(const __hip_bfloat16* __restrict__ base, long long ld, int r0, int k0, int r_lim, int k_lim,
                                          uint4 (&reg)[8]) {
    const int t = threadIdx.x, c = t & 7, rr = t >> 3;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int r = r0 + rr + 32 * p, k = k0 + 8 * c;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (r < r_lim && k < k_lim) v = *(const uint4*)(base + (long long)r * ld + k);
        reg[p] = v;
    }
}

__device__ __forceinline__ void store_tile(__hip_bfloat16* __restrict__ lds, const uint4 (&reg)[8]) {
    const int t = threadIdx.x, c = t & 7, rr = t >> 3;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int r = rr + 32 * p;
        *(uint4*)(lds + r * BK + ((c ^ ((r >> 1) & 7)) * 8)) = reg[p];
    }
}

__device__ __forceinline__ bf16x8 read_frag(const __hip_bfloat16* __restrict__ lds, int row, int chunk) {
    return *(const bf16x8*)(lds + row * BK + ((chunk ^ ((row >> 1) & 7)) * 8));
}

__global__ __launch_bounds__(256) void gemm_bf16_nt_kernel(Args g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __hip_bfloat16* As = (__hip_bfloat16*)smem;                 // [2][BM*BK]
    __hip_bfloat16* Bs = As + 2 * BM * BK;                      // [2][BN*BK]

    int z, tm, tn;
    if (!work_item(g, z, tm, tn)) return;
    const int m0 = tm * BM, n0 = tn * BN;

    const int z1 = z / g.batch_inner, z2 = z % g.batch_inner;
    const __hip_bfloat16* A = g.A + z1 * g.sA1 + z2 * g.sA2;
    const __hip_bfloat16* B = g.B + z1 * g.sB1 + z2 * g.sB2;

    // the contraction axis may be a concatenation of equal segments (kseg > 0); the causal limit applies inside each
    const int seg_len = g.kseg > 0 ? g.kseg : g.K;
    const int nseg = g.kseg > 0 ? g.K / g.kseg : 1;
    int kend = seg_len;
    if (g.flags & TBOA_GEMM_CAUSAL_K) kend = min(kend, n0 + BN);
    const int nk_seg = (kend + BK - 1) / BK;
    const int nk = nk_seg * nseg;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
    const int l32 = lane & 31, lh = lane >> 5;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    uint4 ra[8], rb[8];
    if (nk > 0) {
        load_tile(A, g.lda, m0, 0, g.M, kend, ra);
        load_tile(B, g.ldb, n0, 0, g.N, kend, rb);   // first tile of segment 0
        store_tile(As, ra);
        store_tile(Bs, rb);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const __hip_bfloat16* a_s = As + cur * BM * BK;
        const __hip_bfloat16* b_s = Bs + cur * BN * BK;
        if (kt + 1 < nk) {
            const int sg = (kt + 1) / nk_seg, kb = sg * seg_len;
            const int k0 = kb + ((kt + 1) - sg * nk_seg) * BK;
            load_tile(A, g.lda, m0, k0, g.M, kb + kend, ra);
            load_tile(B, g.ldb, n0, k0, g.N, kb + kend, rb);
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[4], bfr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) af[i] = read_frag(a_s, wm + 32 * i + l32, 2 * ks + lh);
#pragma unroll
            for (int j = 0; j < 4; ++j) bfr[j] = read_frag(b_s, wn + 32 * j + l32, 2 * ks + lh);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            store_tile(As + (cur ^ 1) * BM * BK, ra);
            store_tile(Bs + (cur ^ 1) * BN * BK, rb);
        }
        __syncthreads();
    }

    // accumulator v of tile (i, j): row 32 i + 8 (v / 4) + 4 (lane / 32) + v % 4, column 32 j + lane % 32
    const long long coff = z1 * g.sC1 + z2 * g.sC2;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lh + (v & 3);
            if (row >= g.M) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = n0 + wn + 32 * j + l32;
                if (col >= g.N) continue;
                const long long idx = coff + (long long)row * g.ldc + col;
                float r = g.alpha * acc[i][j][v];
                if (g.c_bf16) ((__hip_bfloat16*)g.C)[idx] = __float2bfloat16(r);
                else { float* c = (float*)g.C + idx; if (g.accumulate) r += *c; *c = r; }
            }
        }
}

// ------------------------------------------------------------------------------------------------
// Fast path (K a multiple of 32): same tiling, but global memory is copied straight into LDS by
// global_load_lds_dwordx4 (no staging registers, no ds_write) through a ring of 4 stages of 32 k each, so that
// loads for stage kt+3 are in flight while stage kt is multiplied: three stage-times (about 3 x 1024 MFMA cycles) to
// cover HBM latency, against one with the register-staged pipeline above.
// An LDS-direct wavefront load writes lane p's 16 bytes at base + 16 p: a 1 KB block = 16 rows x 64 bytes.  Lane p
// therefore fetches, for row p / 4, the logical chunk (p % 4) ^ ((row / 4) % 4): the XOR swizzle (four rows fill one
// 256-byte bank line here) is applied on the global side.  Rows beyond M or N are clamped (their products are never stored).
constexpr int FK = 32;
constexpr int STAGE_ELEMS = (BM + BN) * FK;     // bf16 elements per stage: A tile then B tile

// One stage = 8 LDS-direct loads per wavefront (4 blocks of the A tile, 4 of the B tile).  The per-lane byte offsets
// are loop-invariant; the tile's k position lives in the uniform base pointers; M0 carries the LDS address of the
// 1 KB block.  Written as inline assembly so that the compiler does not pair every later LDS read with a wait for
// ALL outstanding loads (it cannot tell that the ring slot being filled is not the one being read); the explicit
// s_waitcnt vmcnt(N) + barrier in the main loop is the synchronisation.
__device__ __forceinline__ void lds_direct_16(unsigned voff, const char* base, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2" ::"v"(voff), "s"(lds_addr), "s"(base) : "memory", "m0");
}

__device__ __forceinline__ bf16x8 read_frag32(const __hip_bfloat16* __restrict__ t, int row, int chunk) {
    return *(const bf16x8*)(t + row * FK + ((chunk ^ ((row >> 2) & 3)) * 8));
}

// WAVES = 8: 512 threads, two wavefronts per SIMD, each owning 128 x 64 of the tile (128 accumulators, at most 256
// registers).  With one wavefront per SIMD every cycle it spends issuing an LDS read or an LDS-direct load is a cycle
// in which no MFMA is issued; with two, one wavefront's issue stalls fall into the shadow of the other's MFMAs.
template <int N>
__device__ __forceinline__ void wait_loads_but() { asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(N) : "memory"); }

// NS: stages in the LDS ring (NS - 1 of them in flight while one is multiplied)
template <int WAVES, int NS>
__global__ __launch_bounds__(WAVES * 64) void gemm_bf16_nt_fast_kernel(Args g) {
    constexpr int TJ = (WAVES == 8) ? 2 : 4;         // 32-wide MFMA tile columns per wavefront
    constexpr int LPW = 16 / WAVES;                  // 1 KB blocks of the A tile (and of the B tile) per wavefront and stage
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    __hip_bfloat16* ring = (__hip_bfloat16*)smem;     // [NS][STAGE_ELEMS]

    const bool causal = g.flags & TBOA_GEMM_CAUSAL_K;
    int z, tm, tn;
    if (!work_item(g, z, tm, tn)) return;
    const int m0 = tm * BM, n0 = tn * BN;

    const int z1 = z / g.batch_inner, z2 = z % g.batch_inner;
    const __hip_bfloat16* A = g.A + z1 * g.sA1 + z2 * g.sA2;
    const __hip_bfloat16* B = g.B + z1 * g.sB1 + z2 * g.sB2;

    const int seg_len = g.kseg > 0 ? g.kseg : g.K;
    const int nseg = g.kseg > 0 ? g.K / g.kseg : 1;
    int kend = seg_len;
    if (causal) kend = min(kend, n0 + BN);
    const int nk_seg = kend / FK;                  // kend is a multiple of 32 on this path
    const int nk = nk_seg * nseg;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave / (WAVES / 2)) * 128, wn = (wave % (WAVES / 2)) * (32 * TJ);
    const int l32 = lane & 31, lh = lane >> 5;

    f32x16 acc[4][TJ];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // loop-invariant per-lane byte offsets of this wavefront's loads of a stage, relative to the tile's first row
    unsigned offA[LPW], offB[LPW];
    {
        const int pr = lane >> 2, ph = lane & 3;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int row = 16 * (wave * LPW + i) + pr;
            const int lc = ph ^ ((row >> 2) & 3);
            offA[i] = (unsigned)(((long long)min(row, g.M - 1 - m0) * g.lda + lc * 8) * 2);
            offB[i] = (unsigned)(((long long)min(row, g.N - 1 - n0) * g.ldb + lc * 8) * 2);
        }
    }
    const char* Arow = (const char*)(A + (long long)m0 * g.lda);
    const char* Brow = (const char*)(B + (long long)n0 * g.ldb);
    // byte offset along k of the next stage to be issued (stages are issued strictly in order), kept incrementally
    long long koff_next = 0; int kin_next = 0;
    auto advance = [&]() { kin_next += FK; koff_next += 2 * FK; if (kin_next == kend) { kin_next = 0; koff_next += 2LL * (seg_len - kend); } };
    const unsigned ring_lds = (unsigned)(unsigned long long)((__attribute__((address_space(3))) void*)ring);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    auto issue = [&](int slot) {
        const long long kb = koff_next;
        advance();
        const unsigned st = ring_lds + (unsigned)(slot * STAGE_ELEMS * 2);
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const unsigned blk = (unsigned)(wave_s * LPW + i) * 1024u;
            lds_direct_16(offA[i], Arow + kb, st + blk);
            lds_direct_16(offB[i], Brow + kb, st + (unsigned)(BM * FK * 2) + blk);
        }
    };
    // Fragments are double-buffered in registers at k-step granularity: while the MFMAs of one k-step run, the
    // fragments of the next k-step are read from LDS; LDS-direct loads are issued one by one between MFMAs.
    bf16x8 fa[2][4], fb[2][TJ];
#define TB_LOAD_FRAGS(SET, SLOT, KS)                                                                        \
    {                                                                                                       \
        const __hip_bfloat16* a_s = ring + (SLOT) * STAGE_ELEMS;                                            \
        const __hip_bfloat16* b_s = a_s + BM * FK;                                                          \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) fa[SET][i] = read_frag32(a_s, wm + 32 * i + l32, 2 * (KS) + lh); \
        _Pragma("unroll") for (int i = 0; i < TJ; ++i) fb[SET][i] = read_frag32(b_s, wn + 32 * i + l32, 2 * (KS) + lh); \
    }
#define TB_MMA(SET)                                                                                         \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                           \
        _Pragma("unroll") for (int jj = 0; jj < TJ; ++jj)                                                   \
            acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[SET][i], fb[SET][jj], acc[i][jj], 0, 0, 0);
#define TB_INTERLEAVE_DS                                                                                    \
    __builtin_amdgcn_sched_group_barrier(0x100, 4 + TJ, 0);                                                 \
    __builtin_amdgcn_sched_group_barrier(0x008, 4 * TJ, 0);
    // Stage kt sits in ring slot SLOT, its k-step 0 in register set 0.  Phase 1: read k-step 1 into set 1, multiply
    // set 0.  Phase 2: make stage kt+1 visible (its loads were issued three stages ago), read k-step 0 of stage kt+1
    // into set 0, multiply set 1 and, between the MFMAs, refill slot SLOT (every wavefront has finished reading it)
    // with stage kt+NS.
#define TB_STAGE_STEADY(KT, SLOT, NEXTSLOT)                                                                 \
    {                                                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
        const char* pa_ = Arow + koff_next; const char* pb_ = Brow + koff_next;                             \
        const unsigned st_ = ring_lds + (unsigned)((SLOT) * STAGE_ELEMS * 2);                               \
        advance();                                                                                          \
        TB_LOAD_FRAGS(1, SLOT, 1)                                                                           \
        TB_MMA(0)                                                                                           \
        TB_INTERLEAVE_DS                                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
        wait_loads_but<(NS - 2) * 2 * LPW>();                                                               \
        __syncthreads();                                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
        TB_LOAD_FRAGS(0, NEXTSLOT, 0)                                                                       \
        {                                                                                                   \
            _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                 \
                _Pragma("unroll") for (int jj = 0; jj < TJ; jj += 2) {                                      \
                    acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[1][i], fb[1][jj], acc[i][jj], 0, 0, 0); \
                    acc[i][jj + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[1][i], fb[1][jj + 1], acc[i][jj + 1], 0, 0, 0); \
                    const int q_ = (i * TJ + jj) / 2;              /* 0 .. 2 LPW - 1 */                       \
                    const unsigned blk_ = (unsigned)(wave_s * LPW + q_ / 2) * 1024u;                        \
                    __builtin_amdgcn_sched_barrier(0);                                                      \
                    if (q_ % 2 == 0) lds_direct_16(offA[q_ / 2], pa_, st_ + blk_);                          \
                    else lds_direct_16(offB[q_ / 2], pb_, st_ + (unsigned)(BM * FK * 2) + blk_);            \
                    __builtin_amdgcn_sched_barrier(0);                                                      \
                }                                                                                           \
            }                                                                                               \
        }                                                                                                   \
    }
#define TB_STAGE_TAIL(KT, SLOT, NEXTSLOT)                                                                   \
    {                                                                                                       \
        TB_LOAD_FRAGS(1, SLOT, 1)                                                                           \
        TB_MMA(0)                                                                                           \
        if ((KT) + 1 < nk) {                                                                                \
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");                                     \
            __syncthreads();                                                                                \
            if ((KT) + NS < nk) issue(SLOT);                                                     \
            TB_LOAD_FRAGS(0, NEXTSLOT, 0)                                                                   \
        }                                                                                                   \
        TB_MMA(1)                                                                                           \
    }

    if (nk > 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (s < nk) issue(s);
        if (nk < NS) wait_loads_but<0>();
        else wait_loads_but<(NS - 1) * 2 * LPW>();
        __syncthreads();
        TB_LOAD_FRAGS(0, 0, 0)
        int kt = 0;
        // steady state, unrolled over the ring so that slot numbers are constants: the loads of stages kt+2 and kt+3 may
        // stay in flight while stage kt+1 is awaited
        for (; kt + 2 * NS - 1 < nk; kt += NS) {
#pragma unroll
            for (int u = 0; u < NS; ++u) TB_STAGE_STEADY(kt + u, u, (u + 1) % NS)
        }
        for (; kt < nk; ++kt) TB_STAGE_TAIL(kt, kt % NS, (kt + 1) % NS)
    }
#undef TB_STAGE_STEADY
#undef TB_STAGE_TAIL
#undef TB_MMA
#undef TB_LOAD_FRAGS
#undef TB_INTERLEAVE_DS

    const long long coff = z1 * g.sC1 + z2 * g.sC2;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lh + (v & 3);
            if (row >= g.M) continue;
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                const int col = n0 + wn + 32 * j + l32;
                if (col >= g.N) continue;
                const long long idx = coff + (long long)row * g.ldc + col;
                float r = g.alpha * acc[i][j][v];
                if (g.c_bf16) ((__hip_bfloat16*)g.C)[idx] = __float2bfloat16(r);
                else { float* c = (float*)g.C + idx; if (g.accumulate) r += *c; *c = r; }
            }
        }
}

// Launch order of the output tiles of one batch entry, built once per (tile counts, flags) and kept on the device.
// 32 consecutive tiles run side by side on one XCD, so the order walks compact blocks: row bands of 8 tile rows,
// column by column inside a band (a column's tiles share the B panel, a band's rows the 8 A panels).  A symmetric
// product lists only the tiles on or below the diagonal.  With a causal contraction limit the k-range grows with the
// column, so a band takes its columns from the longest to the shortest (the short ones fill the tail of the launch).
int tile_order(tboa_ctx* ctx, int tiles_m, int tiles_n, int flags, const int** dev, int* count) {
    for (const TileOrder& t : ctx->tile_orders)
        if (t.tiles_m == tiles_m && t.tiles_n == tiles_n && t.flags == flags) { *dev = t.dev; *count = t.count; return 0; }
    const bool lower = flags & TBOA_GEMM_LOWER, causal = flags & TBOA_GEMM_CAUSAL_K;
    const int band = (causal && !lower) ? 16 : 8;
    std::vector<int> h;
    for (int m0 = 0; m0 < tiles_m; m0 += band) {
        const int m1 = m0 + band < tiles_m ? m0 + band : tiles_m;
        for (int c = 0; c < tiles_n; ++c) {
            const int tn = (causal && !lower) ? tiles_n - 1 - c : c;
            for (int tm = m0; tm < m1; ++tm)
                if (!lower || tn <= tm) h.push_back((tm << 16) | tn);
        }
    }
    TileOrder t{tiles_m, tiles_n, flags, nullptr, (int)h.size()};
    TB_HIP(ctx, hipMalloc(&t.dev, h.size() * sizeof(int)));
    hipError_t e = hipMemcpy(t.dev, h.data(), h.size() * sizeof(int), hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(t.dev); return tboa_fail(ctx, TBOA_EHIP, "tile order upload: %s", hipGetErrorString(e)); }
    ctx->tile_orders.push_back(t);
    *dev = t.dev; *count = t.count;
    return 0;
}

}  // namespace

int gemm_bf16_nt(tboa_ctx* ctx, const GemmBf16& q) {
    if (q.M <= 0 || q.N <= 0 || q.batch <= 0) return 0;
    if (!q.A || !q.B || !q.C || q.K < 0) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: null operand or negative K");
    if (q.K % 8 || q.lda % 8 || q.ldb % 8 || ((uintptr_t)q.A & 15) || ((uintptr_t)q.B & 15) || q.strideA % 8 || q.strideB % 8 ||
        q.strideA2 % 8 || q.strideB2 % 8)
        return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: K, leading dimensions and batch strides must be multiples of 8 and pointers 16-byte aligned");
    if (q.c_dtype == TBOA_BF16 && q.accumulate) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: accumulate needs an fp32 C");
    if (q.c_dtype != TBOA_BF16 && q.c_dtype != TBOA_F32) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: C must be fp32 or bf16");
    if ((q.flags & TBOA_GEMM_LOWER) && q.M != q.N) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: LOWER needs M == N");
    static bool attr_set = false;
    const int smem = 2 * (BM + BN) * BK * (int)sizeof(__hip_bfloat16);
    const int smem_fast = 4 * STAGE_ELEMS * (int)sizeof(__hip_bfloat16), smem_fast5 = 5 * STAGE_ELEMS * (int)sizeof(__hip_bfloat16);
    if (!attr_set) {
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_fast_kernel<4, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fast));
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_fast_kernel<8, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fast));
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_fast_kernel<8, 5>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fast5));
        attr_set = true;
    }
    const bool fast = (q.kseg > 0 ? q.kseg : q.K) % FK == 0 && q.K > 0 && !getenv("TBOA_GEMM_GENERIC");
    Args a;
    a.M = q.M; a.N = q.N; a.K = q.K; a.alpha = q.alpha;
    a.A = q.A; a.lda = q.lda; a.B = q.B; a.ldb = q.ldb; a.C = q.C; a.ldc = q.ldc;
    a.c_bf16 = (q.c_dtype == TBOA_BF16); a.accumulate = q.accumulate; a.flags = q.flags;
    a.batch_inner = q.batch_inner > 0 ? q.batch_inner : 1;
    a.kseg = q.kseg;
    if (q.kseg < 0 || (q.kseg > 0 && (q.K % q.kseg || q.kseg % 8))) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: kseg must divide K and be a multiple of 8");
    a.sA1 = q.strideA; a.sB1 = q.strideB; a.sC1 = q.strideC; a.sA2 = q.strideA2; a.sB2 = q.strideB2; a.sC2 = q.strideC2;
    const int tiles_m = (int)cdiv64(q.M, BM), tiles_n = (int)cdiv64(q.N, BN);
    if (tiles_m > 32767 || tiles_n > 32767) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: more than 32767 tiles along one axis");
    TB_TRY(tile_order(ctx, tiles_m, tiles_n, q.flags & (TBOA_GEMM_LOWER | TBOA_GEMM_CAUSAL_K), &a.tile_order, &a.ntiles));
    a.nitems = (long long)a.ntiles * q.batch;
    a.per = (a.nitems + 7) / 8;
    if (a.per > 200000000LL) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: grid too large");
    const unsigned nwg = (unsigned)(8 * a.per);
    const bool timed = ctx->prof_on && q.tag >= 0;
    ProfRec rec{};
    if (timed) {
        TB_HIP(ctx, hipEventCreate(&rec.a)); TB_HIP(ctx, hipEventCreate(&rec.b));
        rec.tag = q.tag;
        const int nseg = q.kseg > 0 ? q.K / q.kseg : 1;
        const double ks = q.kseg > 0 ? q.kseg : q.K;
        double mnk = (double)q.M * q.N * ks;
        if (q.flags & TBOA_GEMM_LOWER) mnk = 0.5 * (double)q.M * (q.M + 1.0) * ks;
        else if ((q.flags & TBOA_GEMM_CAUSAL_K) && ks >= q.N) mnk = 0.5 * (double)q.M * q.N * (q.N + 1.0);
        rec.flops = 2.0 * mnk * nseg * q.batch;
        TB_HIP(ctx, hipEventRecord(rec.a, ctx->stream));
    }
    static const int waves = getenv("TBOA_GEMM_WAVES") ? atoi(getenv("TBOA_GEMM_WAVES")) : 8;
    static const int ring = getenv("TBOA_GEMM_RING") ? atoi(getenv("TBOA_GEMM_RING")) : 4;
    if (fast && waves == 8 && ring == 5) hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<8, 5>), dim3(nwg), dim3(512), smem_fast5, ctx->stream, a);
    else if (fast && waves == 8) hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<8, 4>), dim3(nwg), dim3(512), smem_fast, ctx->stream, a);
    else if (fast) hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<4, 4>), dim3(nwg), dim3(256), smem_fast, ctx->stream, a);
    else hipLaunchKernelGGL(gemm_bf16_nt_kernel, dim3(nwg), dim3(256), smem, ctx->stream, a);
    TB_KERNEL_CHECK(ctx);
    if (timed) { TB_HIP(ctx, hipEventRecord(rec.b, ctx->stream)); ctx->prof.push_back(rec); }
    return 0;
}

extern "C" int tboa_gemm_bf16_nt(tboa_ctx* ctx, int M, int N, int K, float alpha, const void* A, int64_t lda, const void* B,
                                 int64_t ldb, void* C, int64_t ldc, int c_dtype, int accumulate, int flags, int batch,
                                 int64_t strideA, int64_t strideB, int64_t strideC) {
    if (!ctx) return TBOA_EINVAL;
    GemmBf16 g{};
    g.M = M; g.N = N; g.K = K; g.alpha = alpha;
    g.A = (const __hip_bfloat16*)A; g.lda = lda; g.B = (const __hip_bfloat16*)B; g.ldb = ldb;
    g.C = C; g.ldc = ldc; g.c_dtype = c_dtype; g.accumulate = accumulate; g.flags = flags;
    g.batch = batch; g.strideA = strideA; g.strideB = strideB; g.strideC = strideC;
    return gemm_bf16_nt(ctx, g);
}
