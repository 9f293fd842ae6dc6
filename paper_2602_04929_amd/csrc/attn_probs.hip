// Causal attention probabilities of one sequence, written transposed and as (hi, lo) pairs of 16-bit values, straight from
// the operands of the score product: the scores Q_h K_g^T / sqrt(d_h) (Table 1: A_h = softmax of the scaled scores) are
// formed on the matrix cores tile by tile and never stored.  This is what the summed form of the W_V Hessian reads
// (Pt[g][i][r L + t] = A_h[t, i], h = g rep + r; see build_hessians_bf16), for both score matrices at once: the one of the
// quantized-input path and the one of the full-precision path, whose difference A - A~ is the second output.
//
// Operands: Q^ = [q_hi | q_lo | q_hi] and K^ = [k_hi | k_hi | k_lo], one [L, 3 d_h] matrix of 16-bit values per head in 16 x 32
// blocks (as split3_kernel writes them), so that Q^ K^T = q_hi k_hi + q_lo k_hi + q_hi k_lo.  The pairs of a score matrix are
// either IEEE half values of the operands times a power of two (QkScale: 22 significant bits, the products on
// v_mfma_f32_32x32x16_f16 and the powers of two taken back out with the softmax scale) or unscaled bf16 (16 bits).
//
// One workgroup per (128 query rows t, head), eight wavefronts = (path, half of the 64 keys of a tile, half of the queries).
// A wavefront keeps the Q^ fragments of its path for its 64 queries in registers (two 32-wide blocks, the distinct segments q_hi and q_lo)
// and computes S^T = K^ Q^T for its 32 keys: with the keys as the rows of the MFMA result, a lane holds ONE query column
// and 16 key rows, so the running maximum and sum of a query need no traffic between lanes until the end.  The K^ tile of
// both paths (segments k_hi, k_lo: 64 x d_h each) is copied global -> LDS block by block (a 16 x 32 block is 1 KB contiguous
// in memory and lands as it is: its XOR-swizzled 16-byte pieces are what conflict-free fragment reads need), the copy of
// the next tile running under the element-wise work on the current one.
// Pass 1 walks the key tiles up to the diagonal and leaves, per query, maximum and 1 / sum; pass 2 walks them again,
// turns scores into probabilities, exchanges them through LDS (so that A - A~ can be formed and every thread ends up with
// 16 consecutive queries of one key row), and writes whole 16-byte pieces of the blocked result; the key tiles between the
// diagonal and the end of its 256-tile get zeros (a product that starts its contraction at the 256-tile of its rows and
// columns reads nothing else).  Recomputing the scores costs 2 x 3 d_h flops per entry and pass; storing them would cost
// 8 bytes written and 16 read per entry.
#include "internal.h"

typedef __hip_bfloat16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ bf16 enc16(float v, int f16) {
    if (f16) { const _Float16 h = (_Float16)v; return __builtin_bit_cast(bf16, h); }
    return __float2bfloat16(v);
}
__device__ __forceinline__ float dec16(bf16 b, int f16) {
    if (f16) return (float)__builtin_bit_cast(_Float16, b);
    return __bfloat162float(b);
}

constexpr int BT = 128;        // queries per workgroup
// floats per row of the exchange buffer.  Transposed result: the two lane halves of a wavefront write rows 4 apart (4 x 136 = 32 banks
// apart) and the store phase reads 16-byte pieces of a row; row-major result: the store phase reads columns, eight lanes taking rows 8
// apart (8 x 137 = 8 banks apart), the other lanes consecutive queries
template <bool ROWS> constexpr int exch_pitch() { return ROWS ? BT + 9 : BT + 8; }

template <int DH>
constexpr int attn_lds_bytes() { return 4 * 64 * 2 * DH + 2 * 64 * (BT + 9) * 4 + 2 * 2 * 2 * BT * 4 + 2 * 2 * BT * 4; }

// one 1 KB block global -> LDS: lane l moves the 16 bytes at base + voff (voff = 16 l) to lds_addr + 16 l
__device__ __forceinline__ void lds_direct_16(unsigned voff, const char* base, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2" ::"v"(voff), "s"(lds_addr), "s"(base) : "memory", "m0");
}

// 2^x on the transcendental unit
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int DH, bool ROWS>
__global__ __launch_bounds__(512) void attn_probs_t_kernel(const bf16* __restrict__ Qa, const bf16* __restrict__ Ka, const bf16* __restrict__ Qb,
                                                           const bf16* __restrict__ Kb, int L, int nheads, int rep, int xcd_runs, float scale2,
                                                           PtOut out, long long ldp, long long group_stride, int f16, QkScale qs) {
    constexpr int NKS = DH / 16;                 // 16-deep MFMA steps per segment
    constexpr int NCB = DH / 32;                 // 32-column blocks per segment
    constexpr int SEGB = 64 * 2 * DH;            // bytes of one (path, segment) image: [NCB][64 keys][32 elements], pieces swizzled
    constexpr int KB = 3 * DH / 32;              // 16 x 32 blocks per block row of Q^ / K^
    constexpr int NBLK = 2 * 2 * NCB * 4;        // 1 KB blocks of a tile, both paths
    constexpr int EXP = exch_pitch<ROWS>();
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    unsigned char* kt = smem;                                // [path][k_hi, k_lo][NCB][64 keys][64 bytes]
    float* ex = (float*)(smem + 4 * SEGB);                   // [path][64 keys][EXP]: probabilities of the tile
    float* stat = ex + 2 * 64 * EXP;                         // [path][key half][max, sum][BT queries]
    float* fin = stat + 2 * 2 * 2 * BT;                      // [path][max, 1 / sum][BT queries]

    // Work items in the order (KV group, 128-row block from the last, i.e. longest, to the first, head of the group).  When the
    // groups divide evenly over the 8 XCDs (workgroup w runs on XCD w % 8), XCD x takes the contiguous run of items of its
    // groups: the K^ of a group (both paths: 12 L d_h bytes, 3 MB for L = 2048, d_h = 128) then stays in that XCD's L2 and the
    // heads of a group walk the same key tiles side by side.  Otherwise the items are taken in order.
    const int ntb = L / BT, total = nheads * ntb;
    int item = blockIdx.x;
    if (xcd_runs) item = (blockIdx.x & 7) * (total / 8) + (blockIdx.x >> 3);
    const int g = item / (rep * ntb), rem = item % (rep * ntb), r = rem % rep, h = g * rep + r;
    const int t0 = (ntb - 1 - rem / rep) * BT;
    // eight wavefronts = (path, half of the tile's 64 keys, half of the 128 queries); two per SIMD, so that the element-wise
    // work of one runs under the MFMAs of the other
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, p = wave >> 2, wi = (wave >> 1) & 1, th = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const bool two = Qb != nullptr, active = (p == 0) || two;
    const long long mat = (long long)L * 3 * DH;
    const bf16* K0 = Ka + g * mat; const bf16* K1 = two ? Kb + g * mat : K0;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const unsigned kt_lds = (unsigned)(unsigned long long)((__attribute__((address_space(3))) void*)kt);
    const int tq = t0 + 64 * th;                 // first query of this wavefront
    // encoding of this path's operands (uniform over the wavefront) and the scale that takes their powers of two back out
    bool half_ops = false;
    float sc2 = scale2;
    {
        const int* wq = p ? qs.qb : qs.qa; const int* wk = p ? qs.kb : qs.ka;
        if (active && wq && wk) {
            const int bq = __builtin_amdgcn_readfirstlane(*wq), bk = __builtin_amdgcn_readfirstlane(*wk);
            if (bq >= 0 && bk >= 0) { half_ops = true; sc2 = ldexpf(scale2, -(tboa_half_exp(bq) + tboa_half_exp(bk))); }
        }
    }

    // Q^ fragments of this wavefront's path: B operand of the MFMA (lane: query l32 of block tb, 8 contraction elements from 8 lh)
    bf16x8 qh[2][NKS], ql[2][NKS];
    if (active) {
        const bf16* Qp = (p ? Qb : Qa) + h * mat;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const int t = tq + 32 * tb + l32, c = 16 * ks + 8 * lh;
                qh[tb][ks] = *(const bf16x8*)(Qp + tboa_blocked_offset(t, c, KB));
                ql[tb][ks] = *(const bf16x8*)(Qp + tboa_blocked_offset(t, DH + c, KB));
            }
    }

    // the K^ tile at keys i0: block b = ((path 2 + segment) NCB + cb) 4 + rb of the LDS image comes from block
    // (i0 / 16 + rb, segment's first block + cb) of that path's K^; wavefront w copies the blocks w, w + 8, ...
    auto issue = [&](int i0) {
        const int nblk = two ? NBLK : NBLK / 2;
#pragma unroll
        for (int j = 0; j < NBLK / 8; ++j) {
            const int b = wave_s + 8 * j;
            if (b < nblk) {
                const int rb = b & 3, cb = (b >> 2) % NCB, ps = (b >> 2) / NCB;     // ps = path 2 + segment (k_hi, k_lo)
                const bf16* src = ((ps >> 1) ? K1 : K0) + ((long long)((i0 >> 4) + rb) * KB + ((ps & 1) ? 2 * NCB : 0) + cb) * 512;
                lds_direct_16((unsigned)lane * 16u, (const char*)src, kt_lds + (unsigned)b * 1024u);
            }
        }
    };
    // S^T of the tile for this wavefront: acc[tb][4 b + j] = q . k of (key i0 + 32 wi + 8 b + 4 lh + j, query tq + 32 tb + l32)
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 acc[2];
    auto multiply = [&]() {
        acc[0] = zero16; acc[1] = zero16;
        const int row = 32 * wi + l32;
        const unsigned char* kh_img = kt + (p * 2 + 0) * SEGB + row * 64;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int c8 = 2 * ks + lh;                                   // 8-element piece of the segment
            const int off = (c8 >> 2) * 4096 + (((c8 & 3) ^ ((row >> 2) & 3)) << 4);
            const bf16x8 kh = *(const bf16x8*)(kh_img + off), kl = *(const bf16x8*)(kh_img + SEGB + off);
            if (half_ops) {
                const f16x8 fkh = __builtin_bit_cast(f16x8, kh), fkl = __builtin_bit_cast(f16x8, kl);
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    const f16x8 fqh = __builtin_bit_cast(f16x8, qh[tb][ks]), fql = __builtin_bit_cast(f16x8, ql[tb][ks]);
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fkh, fqh, acc[tb], 0, 0, 0);
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fkh, fql, acc[tb], 0, 0, 0);
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fkl, fqh, acc[tb], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kh, qh[tb][ks], acc[tb], 0, 0, 0);
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kh, ql[tb][ks], acc[tb], 0, 0, 0);
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kl, qh[tb][ks], acc[tb], 0, 0, 0);
                }
            }
        }
    };
    auto landed = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); __syncthreads(); };

    const int live = t0 / 64 + 2;                              // key tiles up to and including the two on the diagonal
    const int tiles = min(L, (t0 / 256 + 1) * 256) / 64;       // ... up to the end of the diagonal's 256-tile
    // Scores are kept in units of log 2: v = (q . k) sc2 with sc2 = log2(e) / sqrt(d_h) (over the operands' powers of two),
    // probabilities 2^(v - max) / sum.
    // ---- pass 1: maximum and sum per query, over this wavefront's keys
    float m[2] = {-INFINITY, -INFINITY}, s[2] = {0.f, 0.f};
    issue(0);
    landed();
    for (int it = 0; it < live; ++it) {
        if (active) multiply();
        __syncthreads();                                   // every wavefront has read the tile
        if (it + 1 < live) issue(64 * (it + 1));           // the next one lands under the element-wise work below
        if (active) {
            const int ib = 64 * it + 32 * wi + 4 * lh;
            const bool masked = 64 * it + 63 > tq;         // a tile that reaches beyond the first query of this wavefront
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int t = tq + 32 * tb + l32;
                float vm = -INFINITY;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    acc[tb][e] *= sc2;
                    if (masked && ib + 8 * (e >> 2) + (e & 3) > t) acc[tb][e] = -INFINITY;
                    vm = fmaxf(vm, acc[tb][e]);
                }
                if (vm > m[tb]) { s[tb] *= ex2(m[tb] - vm); m[tb] = vm; }
                if (m[tb] != -INFINITY) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) s[tb] += ex2(acc[tb][e] - m[tb]);
                }
            }
        }
        landed();
    }
    if (active) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {       // the two lane halves hold different keys of the same query
            const float m2 = __shfl_xor(m[tb], 32, 64), s2 = __shfl_xor(s[tb], 32, 64);
            const float M = fmaxf(m[tb], m2);
            const float sum = (m[tb] == -INFINITY ? 0.f : s[tb] * ex2(m[tb] - M)) + (m2 == -INFINITY ? 0.f : s2 * ex2(m2 - M));
            const int tl = 64 * th + 32 * tb + l32;
            if (lh == 0) { stat[((p * 2 + wi) * 2 + 0) * BT + tl] = M; stat[((p * 2 + wi) * 2 + 1) * BT + tl] = sum; }
        }
    }
    __syncthreads();
    if (threadIdx.x < 2 * BT && (threadIdx.x < BT || two)) {
        const int pp = threadIdx.x / BT, tl = threadIdx.x % BT;
        const float ma = stat[((pp * 2 + 0) * 2 + 0) * BT + tl], sa = stat[((pp * 2 + 0) * 2 + 1) * BT + tl];
        const float mb = stat[((pp * 2 + 1) * 2 + 0) * BT + tl], sb = stat[((pp * 2 + 1) * 2 + 1) * BT + tl];
        const float M = fmaxf(ma, mb);
        const float sum = (ma == -INFINITY ? 0.f : sa * ex2(ma - M)) + (mb == -INFINITY ? 0.f : sb * ex2(mb - M));
        fin[(pp * 2 + 0) * BT + tl] = M; fin[(pp * 2 + 1) * BT + tl] = 1.f / sum;
    }
    __syncthreads();
    float M[2] = {0.f, 0.f}, inv[2] = {0.f, 0.f};
    if (active) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            const int tl = 64 * th + 32 * tb + l32;
            M[tb] = fin[(p * 2 + 0) * BT + tl]; inv[tb] = fin[(p * 2 + 1) * BT + tl];
        }
    }
    // ---- pass 2: probabilities, exchanged through LDS, written transposed.  As IEEE half they are written times 2^14
    // (ATTN_PROBS_HALF_SCALE): the lo half of a pair then stays a normal number down to probabilities of 2^-17, where unscaled it
    // would be subnormal below 2^-3 (an absolute error of 3e-8 on every entry); the products that read them take the factor out.
    const float osc = f16 ? ATTN_PROBS_HALF_SCALE : 1.f;
    bf16* dst[4] = {out.hi + g * group_stride, out.lo ? out.lo + g * group_stride : nullptr, out.dhi ? out.dhi + g * group_stride : nullptr,
                    out.dlo ? out.dlo + g * group_stride : nullptr};
    issue(0);
    landed();
    for (int it = 0; it < tiles; ++it) {
        const int i0 = 64 * it;
        if (it < live) {
            if (active) {
                multiply();
                const int il = 32 * wi + 4 * lh;
                const bool masked = i0 + 63 > tq;
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    const int t = tq + 32 * tb + l32;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int row = il + 8 * (e >> 2) + (e & 3);
                        float a = ex2(acc[tb][e] * sc2 - M[tb]) * inv[tb];
                        if (masked && i0 + row > t) a = 0.f;
                        ex[(p * 64 + row) * EXP + 64 * th + 32 * tb + l32] = a;
                    }
                }
            }
            __syncthreads();                               // the tile has been read, its probabilities are in LDS
            if (it + 1 < live) issue(64 * (it + 1));
        }
        if constexpr (ROWS) {
            // per-head result P[h][t][.] = [A_hi | A_lo | A~_hi | A~_lo] (segments of L columns), queries as rows: eight consecutive
            // lanes take the 64 keys of one query, 8 each; two queries per thread
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int slot = threadIdx.x + 512 * half, i8 = slot & 7, tq2 = slot >> 3;
                union { bf16 b[8]; uint4 u; } hi, lo, h2, l2;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float a = (it < live) ? ex[(8 * i8 + e) * EXP + tq2] * osc : 0.f;
                    const float a2 = (it < live && two) ? ex[(64 + 8 * i8 + e) * EXP + tq2] * osc : 0.f;
                    hi.b[e] = enc16(a, f16); lo.b[e] = enc16(a - dec16(hi.b[e], f16), f16);
                    h2.b[e] = enc16(a2, f16); l2.b[e] = enc16(a2 - dec16(h2.b[e], f16), f16);
                }
                // (the head's [L, ldp] matrix in 16 x 32 blocks: the eight queries of a wavefront store are 512 contiguous bytes per block)
                bf16* ph = out.hi + h * group_stride;
                const long long kb = ldp >> 5, tq3 = t0 + tq2, col = i0 + 8 * i8;
                *(uint4*)(ph + tboa_blocked_offset(tq3, col, kb)) = hi.u; *(uint4*)(ph + tboa_blocked_offset(tq3, L + col, kb)) = lo.u;
                if (two) { *(uint4*)(ph + tboa_blocked_offset(tq3, 2LL * L + col, kb)) = h2.u; *(uint4*)(ph + tboa_blocked_offset(tq3, 3LL * L + col, kb)) = l2.u; }
            }
        } else {
            // transposed blocked result: sixteen consecutive lanes take the 128 queries of one key row, 8 each (one 16-byte piece per
            // output), so that a wavefront store covers four key rows of four blocks, 256 contiguous bytes in each; two rows per thread
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int slot = threadIdx.x + 512 * half, t8 = slot & 15, ri = slot >> 4;
                union { bf16 b[8]; uint4 u; } hi, lo, dh, dl;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    f4 v = {0.f, 0.f, 0.f, 0.f}, w = {0.f, 0.f, 0.f, 0.f};
                    if (it < live) {
                        v = *(const f4*)(ex + ri * EXP + 8 * t8 + 4 * q);
                        if (two) w = *(const f4*)(ex + (64 + ri) * EXP + 8 * t8 + 4 * q);
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float a = v[e] * osc, d = (v[e] - w[e]) * osc;
                        hi.b[4 * q + e] = enc16(a, f16); lo.b[4 * q + e] = enc16(a - dec16(hi.b[4 * q + e], f16), f16);
                        dh.b[4 * q + e] = enc16(d, f16); dl.b[4 * q + e] = enc16(d - dec16(dh.b[4 * q + e], f16), f16);
                    }
                }
                const long long o = tboa_blocked_offset(i0 + ri, (long long)r * L + t0 + 8 * t8, ldp >> 5);
                *(uint4*)(dst[0] + o) = hi.u; *(uint4*)(dst[1] + o) = lo.u;
                if (two) { *(uint4*)(dst[2] + o) = dh.u; *(uint4*)(dst[3] + o) = dl.u; }
            }
        }
        if (it < live) landed();                           // next tile in LDS; the exchange buffer is free again
    }
}

template <int DH, bool ROWS>
int launch(tboa_ctx* ctx, const bf16* Qa, const bf16* Ka, const bf16* Qb, const bf16* Kb, int L, int Hq, int rep, PtOut out, long long ldp,
           long long group_stride, int f16, QkScale qs) {
    static bool attr_set = false;
    constexpr int smem = attn_lds_bytes<DH>();
    if (!attr_set) {
        TB_HIP(ctx, hipFuncSetAttribute((const void*)attn_probs_t_kernel<DH, ROWS>, hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        attr_set = true;
    }
    const int total = Hq * (L / BT), xcd_runs = ((Hq / rep) % 8 == 0 && total % 8 == 0) ? 1 : 0;
    hipLaunchKernelGGL((attn_probs_t_kernel<DH, ROWS>), dim3(total), dim3(512), smem, ctx->stream, Qa, Ka, Qb, Kb, L, Hq, rep, xcd_runs,
                       (float)(1.4426950408889634 / sqrt((double)DH)), out, ldp, group_stride, f16, qs);
    TB_KERNEL_CHECK(ctx);
    return 0;
}

template <bool ROWS>
int dispatch(tboa_ctx* ctx, const bf16* Qa, const bf16* Ka, const bf16* Qb, const bf16* Kb, int L, int Hq, int rep, int dh, PtOut out,
             long long ldp, long long group_stride, int f16, QkScale qs) {
    switch (dh) {
        case 32: return launch<32, ROWS>(ctx, Qa, Ka, Qb, Kb, L, Hq, rep, out, ldp, group_stride, f16, qs);
        case 64: return launch<64, ROWS>(ctx, Qa, Ka, Qb, Kb, L, Hq, rep, out, ldp, group_stride, f16, qs);
        case 96: return launch<96, ROWS>(ctx, Qa, Ka, Qb, Kb, L, Hq, rep, out, ldp, group_stride, f16, qs);
        default: return launch<128, ROWS>(ctx, Qa, Ka, Qb, Kb, L, Hq, rep, out, ldp, group_stride, f16, qs);
    }
}

}  // namespace

bool attn_probs_t_supported(int L, int dh) {
    return L % 256 == 0 && (dh == 32 || dh == 64 || dh == 96 || dh == 128);
}

int attn_probs_t(tboa_ctx* ctx, const bf16* Qa, const bf16* Ka, const bf16* Qb, const bf16* Kb, int L, int Hq, int rep, int dh, PtOut out,
                 long long ldp, long long group_stride, int f16, QkScale qs) {
    if (!attn_probs_t_supported(L, dh) || Hq % rep || !Qa || !Ka || (Qb && !Kb) || !out.hi || !out.lo || (Qb && (!out.dhi || !out.dlo)) || ldp % 32)
        return tboa_fail(ctx, TBOA_EINVAL, "attn_probs_t: unsupported shape or missing buffer");
    return dispatch<false>(ctx, Qa, Ka, Qb, Kb, L, Hq, rep, dh, out, ldp, group_stride, f16, qs);
}

int attn_probs_rows(tboa_ctx* ctx, const bf16* Qa, const bf16* Ka, const bf16* Qb, const bf16* Kb, int L, int Hq, int rep, int dh, bf16* P,
                    long long ldp, int f16, QkScale qs) {
    if (!attn_probs_t_supported(L, dh) || Hq % rep || !Qa || !Ka || (Qb && !Kb) || !P || ldp % 32 || ldp < (Qb ? 4LL : 2LL) * L || ((uintptr_t)P & 15))
        return tboa_fail(ctx, TBOA_EINVAL, "attn_probs_rows: unsupported shape or missing buffer");
    PtOut out{P, nullptr, nullptr, nullptr};
    return dispatch<true>(ctx, Qa, Ka, Qb, Kb, L, Hq, rep, dh, out, ldp, (long long)L * ldp, f16, qs);
}
