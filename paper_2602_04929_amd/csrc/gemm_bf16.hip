// bf16 x bf16 -> fp32 GEMM, C = alpha A B^T, on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16); with TBOA_GEMM_F16 the
// same kernels take IEEE half operands (v_mfma_f32_32x32x16_f16: same layouts, same rate, three more mantissa bits).
//
// Both operands are K-contiguous ("NT"): every contraction of the Hessian build is arranged that way (activations
// are kept in a transposed copy where the token axis is the contraction axis), so one kernel shape serves X^T X,
// the projections, Q K^T, A X and the dominant Y^T Y.
//
// Three kernels share the 256 x 256 output tile per workgroup, the MFMA shape, the epilogue and the order of the tiles:
//   gemm_bf16_nt_fast_kernel  (K a multiple of 32: every launch of the Hessian build and of the grid search) copies global
//                             memory straight into a ring of LDS stages and runs 8 wavefronts; described at its definition;
//   gemm_bf16_nt_stream_kernel (TBOA_GEMM_PERSISTENT, k ranges that are multiples of 128) is the same pipeline run by one
//                             resident workgroup per CU over a list of tiles, the ring streaming across tile boundaries;
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
#include <algorithm>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// one 32 x 32 x 16 matrix-core step on 16-bit operands held as 8 x 16 bits per lane; F16: the bits are IEEE half, else bf16
template <bool F16>
__device__ __forceinline__ f32x16 mma16(bf16x8 a, bf16x8 b, f32x16 c) {
    if constexpr (F16) return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

namespace {

constexpr int BM = 256, BN = 256, BK = 64;

struct Args {
    int M, N, K;
    float alpha;
    const __hip_bfloat16* A; long long lda;
    const __hip_bfloat16* B; long long ldb;
    void* C; long long ldc;
    void* C2;                   // TBOA_GEMM_C_HILO: receives the low parts, same layout as C
    float lo_scale;             // ... times this factor (half pairs: keeps the low parts out of the subnormal range)
    int c_bf16, accumulate, flags;   // c_bf16: C holds 16-bit values (bf16, or IEEE half with TBOA_GEMM_F16)
    int vec_c;                  // C rows and batch offsets allow 16-byte (fp32) / 8-byte (bf16) accesses at columns that are multiples of 4
    int batch_inner, kseg;
    long long sA1, sA2, sB1, sB2, sC1, sC2;
    const int* tile_order;      // (tm << 16 | tn) of the tiles of one batch entry, in launch order
    int ntiles;                 // tiles per batch entry
    long long nitems, per;      // batch * ntiles work items; per = items per XCD
    int chunk;                  // 0: XCD x takes the contiguous run [x per, (x + 1) per); else runs of `chunk` items are dealt to the XCDs in turn
    const int2* sched;          // persistent kernel: [workgroups][rounds] of (batch entry or -1, tm << 16 | tn)
    int rounds;
    // persistent kernel, several operand pairs: after every term_segs segments the operand pointers move on by term_dA /
    // term_dB bytes (the distance to the next pair's buffer less the columns just read); term_segs = 0: one pair
    int term_segs;
    long long term_dA[3], term_dB[3];
};

// Work item of this workgroup.  Workgroups are dealt to the eight XCDs round-robin by their linear number, so workgroup
// w runs on XCD w % 8.  The item list is batch-major, the host-built tile order inside a batch entry.  With a batch of 8
// or more, runs of 32 consecutive items are dealt to the XCDs in turn: the 32 CUs of an XCD work on 32 consecutive tiles
// (a compact block of the output sharing few operand panels through that XCD's L2), and the 256 tiles in flight on the
// chip are consecutive too, so they span two or three batch entries whose operands the memory-side cache can hold
// (measured on the 32-head H_in^V launch: 7.1 -> 6.9 ms against contiguous runs per XCD, where eight heads are in
// flight at once; runs of 16 or 64 items are slower).  Smaller batches: XCD x takes the contiguous run [x per, (x + 1) per).
__device__ __forceinline__ bool work_item(const Args& g, int& z, int& tm, int& tn) {
    const long long loc = blockIdx.x >> 3;
    const long long item = g.chunk ? ((loc / g.chunk) * 8 + (blockIdx.x & 7)) * g.chunk + loc % g.chunk : (long long)(blockIdx.x & 7) * g.per + loc;
    if (loc >= g.per || item >= g.nitems) return false;
    z = (int)(item / g.ntiles);
    const int packed = g.tile_order[(int)(item - (long long)z * g.ntiles)];
    tm = __builtin_amdgcn_readfirstlane(packed >> 16); tn = __builtin_amdgcn_readfirstlane(packed & 0xffff);
    z = __builtin_amdgcn_readfirstlane(z);
    return true;
}

// Epilogue shared by the kernels.  The MFMA leaves lane l of a wavefront with column l % 32 of a 32 x 32 sub-tile and, in
// accumulators 4 b .. 4 b + 3, the four consecutive rows 8 b + 4 (l / 32) + 0 .. 3: stored as they are, that is 128
// wavefront stores of one scalar per lane for a 128 x 64 wavefront tile, twice the number a wavefront can have in flight,
// and the epilogue then runs at the latency of its own stores (9 - 13 us per 256 x 256 tile measured, a third of a short
// causal tile).  transpose_acc swaps rows and columns inside every 4 x 4 block held by four neighbouring lanes (two
// butterfly steps of quad-permute moves), after which lane l holds, for row 8 b + 4 (l / 32) + l % 4, the four consecutive
// columns 4 ((l % 32) / 4) + 0 .. 3: one 16-byte (fp32) or 8-byte (bf16) store per lane and group, eight full rows of
// 128 bytes per wavefront store, 32 stores per wavefront tile.
template <int CTRL>
__device__ __forceinline__ float quad_perm(float v) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}

template <int TJ>
__device__ __forceinline__ void transpose_acc(f32x16 (&acc)[4][TJ]) {
    const bool x0 = threadIdx.x & 1, x1 = threadIdx.x & 2;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                float a0 = acc[i][j][4 * b], a1 = acc[i][j][4 * b + 1], a2 = acc[i][j][4 * b + 2], a3 = acc[i][j][4 * b + 3];
                // with lane ^ 1 (quad_perm [1,0,3,2]): 2 x 2 blocks
                const float r01 = quad_perm<0xB1>(x0 ? a0 : a1), r23 = quad_perm<0xB1>(x0 ? a2 : a3);
                a0 = x0 ? r01 : a0; a1 = x0 ? a1 : r01; a2 = x0 ? r23 : a2; a3 = x0 ? a3 : r23;
                // with lane ^ 2 (quad_perm [2,3,0,1])
                const float r02 = quad_perm<0x4E>(x1 ? a0 : a2), r13 = quad_perm<0x4E>(x1 ? a1 : a3);
                a0 = x1 ? r02 : a0; a2 = x1 ? a2 : r02; a1 = x1 ? r13 : a1; a3 = x1 ? a3 : r13;
                acc[i][j][4 * b] = a0; acc[i][j][4 * b + 1] = a1; acc[i][j][4 * b + 2] = a2; acc[i][j][4 * b + 3] = a3;
            }
}

// acc as left by transpose_acc; (row0, col0): first row and column of the wavefront's tile in C, uniform over the wavefront
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// whether the 16-bit results are IEEE half: single values follow the operands (TBOA_GEMM_F16), (hi, lo) pairs their own flag
__device__ __forceinline__ bool half_results(const Args& g) {
    return (g.flags & TBOA_GEMM_C_HILO) ? (g.flags & TBOA_GEMM_C_HILO_HALF) != 0 : (g.flags & TBOA_GEMM_F16) != 0;
}
// four results as 16-bit values (8 bytes)
__device__ __forceinline__ uint2 pack16x4(const Args& g, f32x4 r) {
    if (half_results(g)) return __builtin_bit_cast(uint2, __builtin_convertvector(r, f16x4));
    return __builtin_bit_cast(uint2, __builtin_convertvector(r, bf16x4));
}
// TBOA_GEMM_C_HILO: the result leaves as a (hi, lo) pair of 16-bit values, hi into C and lo = r - hi (rounded) into C2
__device__ __forceinline__ uint2 pack_lo4(const Args& g, f32x4 r) {
    if (g.flags & TBOA_GEMM_C_HILO_HALF) {
        const f16x4 hi = __builtin_convertvector(r, f16x4);
        return __builtin_bit_cast(uint2, __builtin_convertvector((r - __builtin_convertvector(hi, f32x4)) * g.lo_scale, f16x4));
    }
    const bf16x4 hi = __builtin_convertvector(r, bf16x4);
    return __builtin_bit_cast(uint2, __builtin_convertvector(r - __builtin_convertvector(hi, f32x4), bf16x4));
}

template <int TJ, bool SCALE>
__device__ __forceinline__ void store_acc_interior(const Args& g, const f32x16 (&acc)[4][TJ], int row0, int col0, long long coff) {
    // the whole wavefront tile lies inside C and C allows vector accesses: no predicates, addresses = uniform base of the
    // group + one per-lane offset computed once
    const int lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5;
    const int es = g.c_bf16 ? 2 : 4;
    const unsigned off = (unsigned)(((long long)(4 * lh + (l32 & 3)) * g.ldc + 4 * (l32 >> 2)) * es);
    char* base = (char*)g.C + (coff + (long long)row0 * g.ldc + col0) * es;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                char* p = base + ((long long)(32 * i + 8 * b) * g.ldc + 32 * j) * es + off;
                f32x4 r = {acc[i][j][4 * b], acc[i][j][4 * b + 1], acc[i][j][4 * b + 2], acc[i][j][4 * b + 3]};
                if (SCALE) r *= g.alpha;
                if (g.c_bf16) {
                    *(uint2*)p = pack16x4(g, r);
                    if (g.flags & TBOA_GEMM_C_HILO) *(uint2*)((char*)g.C2 + (p - (char*)g.C)) = pack_lo4(g, r);
                }
                else {
                    if (g.accumulate) r += *(const f32x4*)p;
                    *(f32x4*)p = r;
                }
            }
}

// C in 16 x 32 blocks (TBOA_GEMM_C_TILED; bf16, whole tiles): the 8 bytes of a lane go to row (8 b + 4 (l / 32) + l % 4) % 16
// of block (row / 16, column / 32), piece ((l % 32) / 8) ^ ((row % 16) / 4) of that row, first or second half of the piece
template <int TJ, bool SCALE>
__device__ __forceinline__ void store_acc_tiled(const Args& g, const f32x16 (&acc)[4][TJ], int row0, int col0, long long coff) {
    const int lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5, q = l32 & 3, c = l32 >> 2;
    const long long kb = g.ldc >> 5;
    __hip_bfloat16* base = (__hip_bfloat16*)g.C + coff + ((long long)(row0 >> 4) * kb + (col0 >> 5)) * 512;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int ri = 8 * (b & 1) + 4 * lh + q, cs = (c >> 1) ^ ((2 * (b & 1) + lh) & 3);
            const unsigned off = (unsigned)(ri * 32 + cs * 8 + (c & 1) * 4);
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                f32x4 r = {acc[i][j][4 * b], acc[i][j][4 * b + 1], acc[i][j][4 * b + 2], acc[i][j][4 * b + 3]};
                if (SCALE) r *= g.alpha;
                __hip_bfloat16* p = base + ((long long)(2 * i + (b >> 1)) * kb + j) * 512 + off;
                *(uint2*)p = pack16x4(g, r);
                if (g.flags & TBOA_GEMM_C_HILO) *(uint2*)((__hip_bfloat16*)g.C2 + (p - (__hip_bfloat16*)g.C)) = pack_lo4(g, r);
            }
        }
}

template <int TJ>
__device__ __forceinline__ void store_acc(const Args& g, const f32x16 (&acc)[4][TJ], int row0, int col0, long long coff) {
    if (g.flags & TBOA_GEMM_C_TILED) {
        if (g.alpha == 1.0f) store_acc_tiled<TJ, false>(g, acc, row0, col0, coff);
        else store_acc_tiled<TJ, true>(g, acc, row0, col0, coff);
        return;
    }
    if (g.vec_c && row0 + 128 <= g.M && col0 + 32 * TJ <= g.N) {
        if (g.alpha == 1.0f) store_acc_interior<TJ, false>(g, acc, row0, col0, coff);
        else store_acc_interior<TJ, true>(g, acc, row0, col0, coff);
        return;
    }
    const int lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int row = row0 + 32 * i + 8 * b + 4 * lh + (l32 & 3);
            if (row >= g.M) continue;
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                const int col = col0 + 32 * j + 4 * (l32 >> 2);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (col + e >= g.N) continue;
                    const long long idx = coff + (long long)row * g.ldc + col + e;
                    const float r = g.alpha * acc[i][j][4 * b + e];
                    if (g.c_bf16) {
                        if (g.flags & TBOA_GEMM_C_HILO_HALF) {
                            const _Float16 hi = (_Float16)r;
                            ((_Float16*)g.C)[idx] = hi; ((_Float16*)g.C2)[idx] = (_Float16)((r - (float)hi) * g.lo_scale);
                        } else if (g.flags & TBOA_GEMM_C_HILO) {
                            const __hip_bfloat16 hi = __float2bfloat16(r);
                            ((__hip_bfloat16*)g.C)[idx] = hi; ((__hip_bfloat16*)g.C2)[idx] = __float2bfloat16(r - __bfloat162float(hi));
                        } else if (g.flags & TBOA_GEMM_F16) ((_Float16*)g.C)[idx] = (_Float16)r;
                        else ((__hip_bfloat16*)g.C)[idx] = __float2bfloat16(r);
                    }
                    else { float* c = (float*)g.C + idx; *c = g.accumulate ? r + *c : r; }
                }
            }
        }
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

template <bool F16>
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
    const int kbeg = (g.flags & TBOA_GEMM_KLO) ? min(kend, max(m0, n0)) : 0;      // a multiple of the tile size
    const int nk_seg = (kend - kbeg + BK - 1) / BK;
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
        load_tile(A, g.lda, m0, kbeg, g.M, kend, ra);
        load_tile(B, g.ldb, n0, kbeg, g.N, kend, rb);   // first tile of segment 0
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
            const int k0 = kb + kbeg + ((kt + 1) - sg * nk_seg) * BK;
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
                    acc[i][j] = mma16<F16>(af[i], bfr[j], acc[i][j]);
        }
        if (kt + 1 < nk) {
            store_tile(As + (cur ^ 1) * BM * BK, ra);
            store_tile(Bs + (cur ^ 1) * BN * BK, rb);
        }
        __syncthreads();
    }

    transpose_acc<4>(acc);
    store_acc<4>(g, acc, m0 + __builtin_amdgcn_readfirstlane(wm), n0 + __builtin_amdgcn_readfirstlane(wn), z1 * g.sC1 + z2 * g.sC2);
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
template <int WAVES, int NS, bool F16>
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
    const int kbeg = (g.flags & TBOA_GEMM_KLO) ? min(kend, max(m0, n0)) : 0;      // a multiple of the tile size
    const int nk_seg = (kend - kbeg) / FK;         // kend is a multiple of 32 on this path
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
    const bool tiledA = g.flags & TBOA_GEMM_A_TILED, tiledB = g.flags & TBOA_GEMM_B_TILED;
    const int shA = tiledA ? 4 : 0, shB = tiledB ? 4 : 0;
    unsigned offA[LPW], offB[LPW];
    {
        const int pr = lane >> 2, ph = lane & 3;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int row = 16 * (wave * LPW + i) + pr;
            const int lc = ph ^ ((row >> 2) & 3);
            offA[i] = (unsigned)(((long long)min(row, g.M - 1 - m0) * g.lda + lc * 8) * 2);
            offB[i] = (unsigned)(((long long)min(row, g.N - 1 - n0) * g.ldb + lc * 8) * 2);
            // an operand stored in 16 x 32 blocks: block row of the 1 KB block, the lane's 16 bytes inside it
            if (tiledA) offA[i] = (unsigned)((long long)min(wave * LPW + i, (g.M - 1 - m0) >> 4) * (g.lda >> 5) * 1024 + lane * 16);
            if (tiledB) offB[i] = (unsigned)((long long)min(wave * LPW + i, (g.N - 1 - n0) >> 4) * (g.ldb >> 5) * 1024 + lane * 16);
        }
    }
    // (for a blocked operand m0 * lda is also the element offset of its block row m0 / 16)
    const char* Arow = (const char*)(A + (long long)m0 * g.lda);
    const char* Brow = (const char*)(B + (long long)n0 * g.ldb);
    // byte offset along k of the next stage to be issued (stages are issued strictly in order), kept incrementally;
    // in a blocked operand 32 k are one block of 1 KB, not 64 bytes of a row
    long long koff_next = 2LL * kbeg; int kin_next = kbeg;
    auto advance = [&]() { kin_next += FK; koff_next += 2 * FK; if (kin_next == kend) { kin_next = kbeg; koff_next += 2LL * (seg_len - kend + kbeg); } };
    const unsigned ring_lds = (unsigned)(unsigned long long)((__attribute__((address_space(3))) void*)ring);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    auto issue = [&](int slot) {
        const long long kb = koff_next;
        advance();
        const unsigned st = ring_lds + (unsigned)(slot * STAGE_ELEMS * 2);
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const unsigned blk = (unsigned)(wave_s * LPW + i) * 1024u;
            lds_direct_16(offA[i], Arow + (kb << shA), st + blk);
            lds_direct_16(offB[i], Brow + (kb << shB), st + (unsigned)(BM * FK * 2) + blk);
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
            acc[i][jj] = mma16<F16>(fa[SET][i], fb[SET][jj], acc[i][jj]);
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
        const char* pa_ = Arow + (koff_next << shA); const char* pb_ = Brow + (koff_next << shB);           \
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
                    acc[i][jj] = mma16<F16>(fa[1][i], fb[1][jj], acc[i][jj]); \
                    acc[i][jj + 1] = mma16<F16>(fa[1][i], fb[1][jj + 1], acc[i][jj + 1]); \
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

    transpose_acc<TJ>(acc);
    store_acc<TJ>(g, acc, m0 + __builtin_amdgcn_readfirstlane(wm), n0 + __builtin_amdgcn_readfirstlane(wn), z1 * g.sC1 + z2 * g.sC2);
}

// ------------------------------------------------------------------------------------------------
// Persistent form of the fast path: one workgroup per CU walks a host-built list of tiles (tile_schedule below) and the
// ring of LDS stages runs as ONE stream of stages across tile boundaries.  While the last three stages of a tile are
// multiplied the first three of the next tile are already being fetched, every stage of every tile takes the steady
// path, and no workgroup is dispatched per tile: a dispatched 512-thread workgroup with 128 KB of LDS costs about
// 0.4 us of its XCD's dispatcher (4096 empty ones take 0.2 ms), which together with the exposed ring fill and drain was
// 12 - 15 us per tile, a third of the time of the short causal A X tiles.
// Needs every tile's stage count to be a multiple of NS (k ranges that are multiples of 32 NS), so that tile boundaries
// fall on the boundaries of the unrolled ring.  After the last stage of the list the stream keeps re-reading its final
// stage (in bounds, never multiplied), so the count of outstanding loads a wait refers to never changes.
template <int NS, bool F16>
__global__ __launch_bounds__(512) void gemm_bf16_nt_stream_kernel(Args g) {
    constexpr int TJ = 2, LPW = 2;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    __hip_bfloat16* ring = (__hip_bfloat16*)smem;     // [NS][STAGE_ELEMS]

    const bool causal = g.flags & TBOA_GEMM_CAUSAL_K;
    const int2* __restrict__ my = g.sched + (long long)blockIdx.x * g.rounds;
    const int seg_len = g.kseg > 0 ? g.kseg : g.K;
    const int nseg = g.kseg > 0 ? g.K / g.kseg : 1;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave / 4) * 128, wn = (wave % 4) * 64;
    const int l32 = lane & 31, lh = lane >> 5;

    // a tile of the list, decoded: everything here is uniform over the workgroup
    struct Tile { int valid, m0, n0, kbeg, kend, nk; const char *A, *B; long long coff; };
    auto decode = [&](int2 e) {
        Tile t;
        t.valid = e.x >= 0;
        const int z = t.valid ? e.x : 0;
        t.m0 = (e.y >> 16) * BM; t.n0 = (e.y & 0xffff) * BN;
        const int z1 = z / g.batch_inner, z2 = z % g.batch_inner;
        t.A = (const char*)(g.A + z1 * g.sA1 + z2 * g.sA2 + (long long)t.m0 * g.lda);
        t.B = (const char*)(g.B + z1 * g.sB1 + z2 * g.sB2 + (long long)t.n0 * g.ldb);
        t.coff = z1 * g.sC1 + z2 * g.sC2;
        t.kend = causal ? min(seg_len, t.n0 + BN) : seg_len;
        t.kbeg = (g.flags & TBOA_GEMM_KLO) ? min(t.kend, max(t.m0, t.n0)) : 0;
        t.nk = (t.kend - t.kbeg) / FK * nseg;
        return t;
    };
    const int2 none = make_int2(-1, 0);
    Tile cur = decode(my[0]);
    if (!cur.valid) return;
    Tile nxt = decode(g.rounds > 1 ? my[1] : none);
    int2 raw2 = g.rounds > 2 ? my[2] : none;
    int t_idx = 0;

    // the stream of stages being fetched: position inside the tile it is in
    const bool tiledA = g.flags & TBOA_GEMM_A_TILED, tiledB = g.flags & TBOA_GEMM_B_TILED;     // operands in 16 x 32 blocks
    const int shA = tiledA ? 4 : 0, shB = tiledB ? 4 : 0;
    unsigned offA[LPW], offB[LPW];
    auto set_offsets = [&](int m0, int n0) {
        const int pr = lane >> 2, ph = lane & 3;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int row = 16 * (wave * LPW + i) + pr;
            const int lc = ph ^ ((row >> 2) & 3);
            offA[i] = (unsigned)(((long long)min(row, g.M - 1 - m0) * g.lda + lc * 8) * 2);
            offB[i] = (unsigned)(((long long)min(row, g.N - 1 - n0) * g.ldb + lc * 8) * 2);
            if (tiledA) offA[i] = (unsigned)((long long)min(wave * LPW + i, (g.M - 1 - m0) >> 4) * (g.lda >> 5) * 1024 + lane * 16);
            if (tiledB) offB[i] = (unsigned)((long long)min(wave * LPW + i, (g.N - 1 - n0) >> 4) * (g.ldb >> 5) * 1024 + lane * 16);
        }
    };
    const char* sA = cur.A; const char* sB = cur.B;
    long long koff = 2LL * cur.kbeg; int kin = cur.kbeg, skbeg = cur.kbeg, skend = cur.kend, sleft = cur.nk;
    int sseg = 0, sterm = 0;      // segments read of the current operand pair, and its number
    bool nxt_taken = false;
    set_offsets(cur.m0, cur.n0);
    // called after the loads of the stage the stream points to have been issued
    auto advance = [&]() {
        if (sleft == 0) return;
        if (--sleft > 0) {
            kin += FK; koff += 2 * FK;
            if (kin == skend) {
                kin = skbeg; koff += 2LL * (seg_len - skend + skbeg);
                if (g.term_segs && ++sseg == g.term_segs) { sA += g.term_dA[sterm]; sB += g.term_dB[sterm]; ++sterm; sseg = 0; }
            }
        } else if (nxt.valid && !nxt_taken) {
            sA = nxt.A; sB = nxt.B; skbeg = nxt.kbeg; skend = nxt.kend; sleft = nxt.nk; koff = 2LL * nxt.kbeg; kin = nxt.kbeg;
            sseg = 0; sterm = 0;
            set_offsets(nxt.m0, nxt.n0);
            nxt_taken = true;
        }
    };
    const unsigned ring_lds = (unsigned)(unsigned long long)((__attribute__((address_space(3))) void*)ring);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);

    f32x16 acc[4][TJ];
    bf16x8 fa[2][4], fb[2][TJ];
#define TB_LOAD_FRAGS(SET, SLOT, KS)                                                                        \
    {                                                                                                       \
        const __hip_bfloat16* a_s = ring + (SLOT) * STAGE_ELEMS;                                            \
        const __hip_bfloat16* b_s = a_s + BM * FK;                                                          \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) fa[SET][i] = read_frag32(a_s, wm + 32 * i + l32, 2 * (KS) + lh); \
        _Pragma("unroll") for (int i = 0; i < TJ; ++i) fb[SET][i] = read_frag32(b_s, wn + 32 * i + l32, 2 * (KS) + lh); \
    }
    // one stage: as in gemm_bf16_nt_fast_kernel, except that the loads issued between the MFMAs of phase 2 belong to the
    // stream's position, which may already be in the next tile
#define TB_STAGE(SLOT, NEXTSLOT, WAIT, FIRST)                                                               \
    {                                                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
        const char* pa_ = sA + (koff << shA); const char* pb_ = sB + (koff << shB);                         \
        const unsigned st_ = ring_lds + (unsigned)((SLOT) * STAGE_ELEMS * 2);                               \
        TB_LOAD_FRAGS(1, SLOT, 1)                                                                           \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                       \
            _Pragma("unroll") for (int jj = 0; jj < TJ; ++jj)                                               \
                acc[i][jj] = mma16<F16>(fa[0][i], fb[0][jj], (FIRST) ? zero16 : acc[i][jj]); \
        __builtin_amdgcn_sched_group_barrier(0x100, 4 + TJ, 0);                                             \
        __builtin_amdgcn_sched_group_barrier(0x008, 4 * TJ, 0);                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
        if (WAIT) wait_loads_but<(NS - 2) * 2 * LPW>();                                                     \
        else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                             \
        __syncthreads();                                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
        TB_LOAD_FRAGS(0, NEXTSLOT, 0)                                                                       \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                     \
            _Pragma("unroll") for (int jj = 0; jj < TJ; jj += 2) {                                          \
                acc[i][jj] = mma16<F16>(fa[1][i], fb[1][jj], acc[i][jj]); \
                acc[i][jj + 1] = mma16<F16>(fa[1][i], fb[1][jj + 1], acc[i][jj + 1]); \
                const int q_ = (i * TJ + jj) / 2;              /* 0 .. 2 LPW - 1 */                           \
                const unsigned blk_ = (unsigned)(wave_s * LPW + q_ / 2) * 1024u;                            \
                __builtin_amdgcn_sched_barrier(0);                                                          \
                if (q_ % 2 == 0) lds_direct_16(offA[q_ / 2], pa_, st_ + blk_);                              \
                else lds_direct_16(offB[q_ / 2], pb_, st_ + (unsigned)(BM * FK * 2) + blk_);                \
                __builtin_amdgcn_sched_barrier(0);                                                          \
            }                                                                                               \
        }                                                                                                   \
        advance();                                                                                          \
    }

    // fill the ring: the first NS stages of the stream
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const unsigned st = ring_lds + (unsigned)(s * STAGE_ELEMS * 2);
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const unsigned blk = (unsigned)(wave_s * LPW + i) * 1024u;
            lds_direct_16(offA[i], sA + (koff << shA), st + blk);
            lds_direct_16(offB[i], sB + (koff << shB), st + (unsigned)(BM * FK * 2) + blk);
        }
        advance();
    }
    wait_loads_but<0>();      // all NS stages: the first tile starts like every other one, with NS - 1 stages known to be there
    __syncthreads();
    TB_LOAD_FRAGS(0, 0, 0)

    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    while (true) {
        const int nk = cur.nk;     // the first MFMAs of the tile start from zero: no pass over the accumulators
        // stages 1 .. NS - 1 of the tile landed before the previous epilogue (or the fill): only the last stage of the first
        // round waits, for stage NS
#pragma unroll
        for (int u = 0; u < NS; ++u) TB_STAGE(u, (u + 1) % NS, u == NS - 1, u == 0)
        for (int kt = NS; kt < nk; kt += NS) {
#pragma unroll
            for (int u = 0; u < NS; ++u) TB_STAGE(u, (u + 1) % NS, true, false)
        }
        transpose_acc<TJ>(acc);
        // every load of the stream issued so far (up to stage NS - 1 of the next tile) has landed before the first store is
        // issued: the first NS - 1 stages of the next tile then need no wait, and by the time stage NS is awaited the stores
        // (which count among the outstanding operations) have had NS - 1 stage times to be acknowledged
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        store_acc<TJ>(g, acc, cur.m0 + __builtin_amdgcn_readfirstlane(wm), cur.n0 + __builtin_amdgcn_readfirstlane(wn), cur.coff);
        if (!nxt.valid) break;
        cur = nxt;                       // the stream entered this tile at least one stage ago
        nxt = decode(raw2); nxt_taken = false;
        ++t_idx;
        raw2 = t_idx + 2 < g.rounds ? my[t_idx + 2] : none;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the re-read stages still in flight write LDS
#undef TB_STAGE
#undef TB_LOAD_FRAGS
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

// Tile lists of the persistent kernel: workgroup w (on XCD w % 8) takes its tiles from XCD (w % 8)'s contiguous run of
// the item list (batch-major, the order above inside a batch entry).  Inside a window of the run (one batch entry, or
// 128 items when entries are small) the tiles go, longest contraction first, each to the workgroup of that XCD with the
// least work so far: with equal tiles that is round-robin (32 consecutive tiles side by side, as with dispatched
// workgroups), with a causal limit it pairs long and short tiles so that all lists end together.
int tile_schedule(tboa_ctx* ctx, const GemmBf16& q, int tiles_m, int tiles_n, const int2** dev, int* rounds, int* wgs) {
    const int flags = q.flags & (TBOA_GEMM_LOWER | TBOA_GEMM_CAUSAL_K | TBOA_GEMM_KLO);
    const int seg_len = (flags & (TBOA_GEMM_CAUSAL_K | TBOA_GEMM_KLO)) ? (q.kseg > 0 ? q.kseg : q.K) : 0;
    for (const TileSchedule& t : ctx->tile_schedules)
        if (t.tiles_m == tiles_m && t.tiles_n == tiles_n && t.flags == flags && t.batch == q.batch && t.seg_len == seg_len) {
            *dev = t.dev; *rounds = t.rounds; *wgs = t.wgs; return 0;
        }
    std::vector<int> order;
    {
        const bool lower = flags & TBOA_GEMM_LOWER, causal = flags & TBOA_GEMM_CAUSAL_K;
        const int band = (causal && !lower) ? 16 : 8;
        for (int m0 = 0; m0 < tiles_m; m0 += band) {
            const int m1 = m0 + band < tiles_m ? m0 + band : tiles_m;
            for (int c = 0; c < tiles_n; ++c) {
                const int tn = (causal && !lower) ? tiles_n - 1 - c : c;
                for (int tm = m0; tm < m1; ++tm)
                    if (!lower || tn <= tm) order.push_back((tm << 16) | tn);
            }
        }
    }
    const long long ntiles = (long long)order.size(), nitems = ntiles * q.batch, per = (nitems + 7) / 8;
    const int wpx = (int)(per < 32 ? per : 32);
    const long long window = ntiles >= 64 ? ntiles : 128;
    std::vector<std::vector<int2>> lists((size_t)8 * wpx);
    auto length = [&](int packed) {      // relative cost of a tile: its contraction range
        if (!seg_len) return 1LL;
        const long long hi = (flags & TBOA_GEMM_CAUSAL_K) ? std::min<long long>(seg_len, ((packed & 0xffff) + 1LL) * BN) : seg_len;
        const long long lo = (flags & TBOA_GEMM_KLO) ? std::min<long long>(hi, (long long)std::max(packed >> 16, packed & 0xffff) * BM) : 0;
        return std::max(1LL, hi - lo);
    };
    for (int x = 0; x < 8; ++x) {
        std::vector<long long> load(wpx, 0);
        const long long lo = x * per, hi = std::min(nitems, lo + per);
        for (long long w0 = lo; w0 < hi; w0 += window) {
            const long long w1 = std::min(hi, w0 + window);
            std::vector<long long> idx;
            for (long long it = w0; it < w1; ++it) idx.push_back(it);
            std::stable_sort(idx.begin(), idx.end(), [&](long long a, long long b) { return length(order[a % ntiles]) > length(order[b % ntiles]); });
            for (long long it : idx) {
                int best = 0;
                for (int c = 1; c < wpx; ++c) if (load[c] < load[best]) best = c;
                load[best] += length(order[it % ntiles]);
                lists[(size_t)best * 8 + x].push_back(make_int2((int)(it / ntiles), order[it % ntiles]));
            }
        }
    }
    size_t r = 1;
    for (auto& l : lists) r = std::max(r, l.size());
    std::vector<int2> h((size_t)8 * wpx * r, make_int2(-1, 0));
    for (size_t w = 0; w < lists.size(); ++w) std::copy(lists[w].begin(), lists[w].end(), h.begin() + w * r);
    TileSchedule t{tiles_m, tiles_n, flags, q.batch, seg_len, nullptr, (int)r, 8 * wpx};
    TB_HIP(ctx, hipMalloc(&t.dev, h.size() * sizeof(int2)));
    hipError_t e = hipMemcpy(t.dev, h.data(), h.size() * sizeof(int2), hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(t.dev); return tboa_fail(ctx, TBOA_EHIP, "tile schedule upload: %s", hipGetErrorString(e)); }
    ctx->tile_schedules.push_back(t);
    *dev = t.dev; *rounds = t.rounds; *wgs = t.wgs;
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
    if (q.flags & (TBOA_GEMM_A_TILED | TBOA_GEMM_B_TILED)) {
        const bool ta = q.flags & TBOA_GEMM_A_TILED, tb = q.flags & TBOA_GEMM_B_TILED;
        if ((q.kseg > 0 ? q.kseg : q.K) % 32 || q.K <= 0) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: blocked operands need K (and kseg) to be multiples of 32");
        // (batch strides only need the 16-byte alignment of every operand: a stride may be the distance between two buffers;
        // blocks that start on 128-byte boundaries are read as whole cache lines)
        if ((ta && (q.lda % 32 || q.M % 16)) || (tb && (q.ldb % 32 || q.N % 16)))
            return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: a blocked operand needs rows % 16 == 0 and ld % 32 == 0");
    }
    if (q.flags & TBOA_GEMM_KLO) {
        const int sl = q.kseg > 0 ? q.kseg : q.K;
        if (sl % 256 || q.M > sl || q.N > sl) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: KLO needs a contraction (segment) length that is a multiple of 256 and at least M and N");
    }
    if (q.flags & TBOA_GEMM_C_HILO) {
        if (q.c_dtype != TBOA_BF16 || !q.C2 || ((uintptr_t)q.C2 & 7)) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: a (hi, lo) result needs a 16-bit C and a second buffer");
    } else if (q.flags & TBOA_GEMM_C_HILO_HALF) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: half pairs are a kind of (hi, lo) result");
    if (q.flags & TBOA_GEMM_C_TILED) {
        if (q.c_dtype != TBOA_BF16 || q.accumulate || q.M % 256 || q.N % 256 || q.ldc % 32 || q.strideC % 4 || q.strideC2 % 4 || ((uintptr_t)q.C & 7))
            return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: a blocked C must be bf16 without accumulation, M and N multiples of 256, ldc a multiple of 32");
    }
    static bool attr_set = false;
    const int smem = 2 * (BM + BN) * BK * (int)sizeof(__hip_bfloat16);
    const int smem_fast = 4 * STAGE_ELEMS * (int)sizeof(__hip_bfloat16);
    if (!attr_set) {
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_fast_kernel<8, 4, false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fast));
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_fast_kernel<8, 4, true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fast));
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_stream_kernel<4, false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fast));
        TB_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bf16_nt_stream_kernel<4, true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_fast));
        attr_set = true;
    }
    const bool fast = (q.kseg > 0 ? q.kseg : q.K) % FK == 0 && q.K > 0;
    if ((q.flags & (TBOA_GEMM_A_TILED | TBOA_GEMM_B_TILED)) && !fast) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: blocked operands are read by the LDS-direct kernel only");
    Args a{};
    a.sched = nullptr; a.rounds = 0;
    a.M = q.M; a.N = q.N; a.K = q.K; a.alpha = q.alpha;
    a.A = q.A; a.lda = q.lda; a.B = q.B; a.ldb = q.ldb; a.C = q.C; a.ldc = q.ldc; a.C2 = q.C2; a.lo_scale = q.lo_scale;
    a.c_bf16 = (q.c_dtype == TBOA_BF16); a.accumulate = q.accumulate; a.flags = q.flags;
    a.vec_c = q.ldc % 4 == 0 && q.strideC % 4 == 0 && q.strideC2 % 4 == 0 && ((uintptr_t)q.C & 15) == 0;
    a.batch_inner = q.batch_inner > 0 ? q.batch_inner : 1;
    a.kseg = q.kseg;
    if (q.kseg < 0 || (q.kseg > 0 && (q.K % q.kseg || q.kseg % 8))) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: kseg must divide K and be a multiple of 8");
    a.sA1 = q.strideA; a.sB1 = q.strideB; a.sC1 = q.strideC; a.sA2 = q.strideA2; a.sB2 = q.strideB2; a.sC2 = q.strideC2;
    const int tiles_m = (int)cdiv64(q.M, BM), tiles_n = (int)cdiv64(q.N, BN);
    if (tiles_m > 32767 || tiles_n > 32767) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: more than 32767 tiles along one axis");
    TB_TRY(tile_order(ctx, tiles_m, tiles_n, q.flags & (TBOA_GEMM_LOWER | TBOA_GEMM_CAUSAL_K), &a.tile_order, &a.ntiles));
    a.nitems = (long long)a.ntiles * q.batch;
    a.per = (a.nitems + 7) / 8;
    a.chunk = 0;
    if (q.batch >= 8) { a.chunk = 32; a.per = ((a.nitems + a.chunk - 1) / a.chunk + 7) / 8 * a.chunk; }
    if (a.per > 200000000LL) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: grid too large");
    const unsigned nwg = (unsigned)(8 * a.per);
    ProfRec rec{}; bool timed = false;
    if (ctx->prof_on && q.tag >= 0) {
        const int nseg = q.kseg > 0 ? q.K / q.kseg : 1;
        const double ks = q.kseg > 0 ? q.kseg : q.K;
        double mnk = (double)q.M * q.N * ks;
        if ((q.flags & TBOA_GEMM_KLO) && q.M == q.N) {      // sum over (i, j) of (ks - max(i, j)); the symmetric product: i >= j only
            const double n = q.M;
            mnk = (q.flags & TBOA_GEMM_LOWER) ? n * ks * (n + 1.0) / 2.0 - (n - 1.0) * n * (n + 1.0) / 3.0
                                              : n * n * ks - (n - 1.0) * n * (4.0 * n + 1.0) / 6.0;
        }
        else if (q.flags & TBOA_GEMM_LOWER) mnk = 0.5 * (double)q.M * (q.M + 1.0) * ks;
        else if ((q.flags & TBOA_GEMM_CAUSAL_K) && ks >= q.N) mnk = 0.5 * (double)q.M * q.N * (q.N + 1.0);
        TB_TRY(prof_begin(ctx, q.tag, 2.0 * mnk * nseg * q.batch, rec, timed));
    }
    const bool f16 = (q.flags & TBOA_GEMM_F16) != 0;
    a.term_segs = 0;
    if (q.nterms > 1) {
        const bool pers = fast && (q.kseg > 0 ? q.kseg : q.K) % (FK * 4) == 0 && (q.flags & TBOA_GEMM_PERSISTENT) != 0;
        const int seg = q.kseg > 0 ? q.kseg : q.K;
        if (!pers || q.nterms > 4 || q.K % q.nterms || (q.K / q.nterms) % seg)
            return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: several operand pairs need the persistent kernel, at most 4 pairs, whole segments per pair");
        const long long term_cols = q.K / q.nterms;
        const long long bytesA = (term_cols * 2) << ((q.flags & TBOA_GEMM_A_TILED) ? 4 : 0), bytesB = (term_cols * 2) << ((q.flags & TBOA_GEMM_B_TILED) ? 4 : 0);
        for (int t = 0; t < q.nterms; ++t)
            if (!q.termA[t] || !q.termB[t] || ((uintptr_t)q.termA[t] & 15) || ((uintptr_t)q.termB[t] & 15))
                return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: operand pair %d missing or not 16-byte aligned", t);
        if (q.termA[0] != q.A || q.termB[0] != q.B) return tboa_fail(ctx, TBOA_EINVAL, "gemm_bf16: the first operand pair must be (A, B)");
        a.term_segs = (int)(term_cols / seg);
        for (int t = 0; t + 1 < q.nterms; ++t) {
            a.term_dA[t] = ((const char*)q.termA[t + 1] - (const char*)q.termA[t]) - bytesA;
            a.term_dB[t] = ((const char*)q.termB[t + 1] - (const char*)q.termB[t]) - bytesB;
        }
    }
    const bool persistent = fast && (q.kseg > 0 ? q.kseg : q.K) % (FK * 4) == 0 && (q.flags & TBOA_GEMM_PERSISTENT) != 0;
    if (persistent) {
        int wgs = 0;
        TB_TRY(tile_schedule(ctx, q, tiles_m, tiles_n, &a.sched, &a.rounds, &wgs));
        if (f16) hipLaunchKernelGGL((gemm_bf16_nt_stream_kernel<4, true>), dim3(wgs), dim3(512), smem_fast, ctx->stream, a);
        else hipLaunchKernelGGL((gemm_bf16_nt_stream_kernel<4, false>), dim3(wgs), dim3(512), smem_fast, ctx->stream, a);
    } else if (fast) {
        if (f16) hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<8, 4, true>), dim3(nwg), dim3(512), smem_fast, ctx->stream, a);
        else hipLaunchKernelGGL((gemm_bf16_nt_fast_kernel<8, 4, false>), dim3(nwg), dim3(512), smem_fast, ctx->stream, a);
    } else if (f16) hipLaunchKernelGGL(gemm_bf16_nt_kernel<true>, dim3(nwg), dim3(256), smem, ctx->stream, a);
    else hipLaunchKernelGGL(gemm_bf16_nt_kernel<false>, dim3(nwg), dim3(256), smem, ctx->stream, a);
    TB_KERNEL_CHECK(ctx);
    TB_TRY(prof_end(ctx, rec, timed));
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
