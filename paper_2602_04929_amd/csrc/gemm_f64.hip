// fp64 GEMM on the CDNA fp64 matrix cores (v_mfma_f64_16x16x4_f64).
//
// C[b] = alpha * A[b] B[b] + beta * C[b].  A(m,k) = A[m*sam + k*sak], B(k,n) = B[k*sbk + n*sbn] with one unit
// stride per operand, so the four transpose cases share one kernel body; the layout of an operand's LDS tile
// follows its contiguous axis so that global loads are coalesced and LDS reads by 16-lane groups are
// conflict-free.  Workgroup: 256 threads = 4 wavefronts (2 x 2), tile 128 x 128 x 16, each wavefront owns a
// 64 x 64 sub-tile as 4 x 4 MFMA tiles (64 fp64 accumulators per lane).  Global -> register -> LDS software
// pipeline with two LDS buffers, one barrier per k-step.
// Products with at most 32 rows per batch entry (the compensation terms of a block of out-channels against a d x d
// factor per head) run a 32 x 128 tile instead (wavefronts 1 x 4, each 32 x 32): with the 128-row tile three quarters
// of the MFMAs would multiply padding, and those products are bound by reading B once from HBM.
#include "internal.h"
#include <algorithm>

typedef double v4d __attribute__((ext_vector_type(4)));

namespace {

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int PKC = BK + 1;   // pitch of a [row][k] tile (k-contiguous operand); odd -> conflict-free 16-lane reads
constexpr int PMC = BM + 16;  // pitch of a [k][row] tile (row-contiguous operand): k and k+1 land 32 of the 64 LDS banks apart
constexpr int TILE = (BM * PKC > BK * PMC) ? BM * PKC : BK * PMC;

struct Args {
    int M, N, K;
    double alpha, beta;
    const double* A; long long sa_r, sa_k;
    const double* B; long long sb_k, sb_r;
    double* C; long long ldc;
    long long strideA, strideB, strideC, strideA2, strideB2, strideC2;
    int batch_inner;
    int klo_m, klo_n, khi_m, khi_n, skip_lower, skip_upper, skip_col0, diag_order;
    const int* m_limit;
    const double* A2; const double* B2;
};

// Loads the BMxBK tile of an operand whose element (r, k) lives at base[r*s_r + k*s_k].
// KC: s_k == 1 (k-contiguous), else s_r == 1.  Out-of-range elements read as zero.
template <bool KC, int ROWS>
__device__ __forceinline__ void load_tile(const double* __restrict__ base, long long s_r, long long s_k,
                                          int r0, int k0, int r_lim, int k_lim, bool vec, double (&reg)[ROWS / 16]) {
    const int t = threadIdx.x;
#pragma unroll
    for (int p = 0; p < ROWS / 32; ++p) {
        const int idx = t + 256 * p;
        int r, k;
        if (KC) { r = idx >> 3; k = (idx & 7) * 2; } else { k = idx / (ROWS / 2); r = (idx % (ROWS / 2)) * 2; }
        const int gr = r0 + r, gk = k0 + k;
        double v0 = 0.0, v1 = 0.0;
        if (KC) {
            if (gr < r_lim) {
                const double* p0 = base + (long long)gr * s_r + gk;
                if (vec && gk + 1 < k_lim) { double2 v = *(const double2*)p0; v0 = v.x; v1 = v.y; }
                else { if (gk < k_lim) v0 = p0[0]; if (gk + 1 < k_lim) v1 = p0[1]; }
            }
        } else {
            if (gk < k_lim) {
                const double* p0 = base + (long long)gk * s_k + gr;
                if (vec && gr + 1 < r_lim) { double2 v = *(const double2*)p0; v0 = v.x; v1 = v.y; }
                else { if (gr < r_lim) v0 = p0[0]; if (gr + 1 < r_lim) v1 = p0[1]; }
            }
        }
        reg[2 * p] = v0; reg[2 * p + 1] = v1;
    }
}

template <bool KC, int ROWS>
__device__ __forceinline__ void store_tile(double* __restrict__ lds, const double (&reg)[ROWS / 16]) {
    const int t = threadIdx.x;
#pragma unroll
    for (int p = 0; p < ROWS / 32; ++p) {
        const int idx = t + 256 * p;
        if (KC) {
            const int r = idx >> 3, k = (idx & 7) * 2;
            lds[r * PKC + k] = reg[2 * p]; lds[r * PKC + k + 1] = reg[2 * p + 1];
        } else {
            const int k = idx / (ROWS / 2), r = (idx % (ROWS / 2)) * 2;
            *(double2*)(lds + k * (ROWS + 16) + r) = make_double2(reg[2 * p], reg[2 * p + 1]);
        }
    }
}

// pitch of a [k][row] tile: ROWS + 16 doubles, so that k and k + 1 land 32 of the 64 LDS banks apart (ROWS = 128 or 32)
template <bool KC, int ROWS>
__device__ __forceinline__ double lds_at(const double* __restrict__ lds, int r, int k) {
    return KC ? lds[r * PKC + k] : lds[k * (ROWS + 16) + r];
}

// TM: rows of the output tile, 128 (wavefronts 2 x 2, 64 x 64 each) or 32 (wavefronts 1 x 4, 32 x 32 each)
template <bool AKC, bool BKC, int TM>
__global__ __launch_bounds__(256) void gemm_f64_kernel(Args g, bool vecA, bool vecB) {
    constexpr int TI = TM == 128 ? 4 : 2, TJ = TM == 128 ? 4 : 2;     // 16 x 16 MFMA tiles per wavefront
    constexpr int ATILE = TM == 128 ? TILE : 32 * (BK + 16);          // covers [32][PKC] and [BK][32 + 16]
    __shared__ __attribute__((aligned(16))) double As[2][ATILE];
    __shared__ __attribute__((aligned(16))) double Bs[2][TILE];

    // Workgroups go to the eight XCDs round-robin by linear number, so with a column count that is a multiple of 8 an XCD
    // always gets the same tile columns; where the contraction length grows with the column (diag_order), the columns of
    // each tile row are rotated by the row number so that every XCD sees all lengths.
    const int tx = g.diag_order ? (int)((blockIdx.x + blockIdx.y) % gridDim.x) : (int)blockIdx.x;
    const int m0 = blockIdx.y * TM, n0 = tx * BN;
    if (g.m_limit && m0 >= g.m_limit[blockIdx.z]) return;
    if (g.skip_lower && g.skip_col0 + n0 + BN <= m0) return;
    if (g.skip_upper && m0 + TM <= g.skip_col0 + n0) return;
    const long long b = blockIdx.z / g.batch_inner, b2 = blockIdx.z % g.batch_inner;
    const double* A = g.A + b * g.strideA + b2 * g.strideA2;
    const double* B = g.B + b * g.strideB + b2 * g.strideB2;
    const double* A2 = g.A2 ? g.A2 + b * g.strideA + b2 * g.strideA2 : nullptr;
    const double* B2 = g.A2 ? g.B2 + b * g.strideB + b2 * g.strideB2 : nullptr;
    double* C = g.C + b * g.strideC + b2 * g.strideC2;

    int klo = 0, khi = g.K;
    if (g.klo_m) klo = max(klo, m0);
    if (g.klo_n) klo = max(klo, n0);
    if (g.khi_m) khi = min(khi, m0 + TM);
    if (g.khi_n) khi = min(khi, n0 + BN);
    klo = (klo / BK) * BK;
    const int nk1 = khi > klo ? (khi - klo + BK - 1) / BK : 0;      // k-steps of one pair of operands
    const int nk = A2 ? 2 * nk1 : nk1;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = TM == 128 ? (wave >> 1) * 64 : 0, wn = TM == 128 ? (wave & 1) * 64 : wave * 32;
    const int l16 = lane & 15, lk = lane >> 4;

    v4d acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) acc[i][j] = (v4d){0.0, 0.0, 0.0, 0.0};

    double ra[TM / 16], rb[8];
    if (nk > 0) {
        load_tile<AKC, TM>(A, g.sa_r, g.sa_k, m0, klo, g.M, khi, vecA, ra);
        load_tile<BKC, BN>(B, g.sb_r, g.sb_k, n0, klo, g.N, khi, vecB, rb);
        store_tile<AKC, TM>(As[0], ra);
        store_tile<BKC, BN>(Bs[0], rb);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            const bool second = kt + 1 >= nk1;
            const int k0 = klo + (kt + 1 - (second ? nk1 : 0)) * BK;
            load_tile<AKC, TM>(second ? A2 : A, g.sa_r, g.sa_k, m0, k0, g.M, khi, vecA, ra);
            load_tile<BKC, BN>(second ? B2 : B, g.sb_r, g.sb_k, n0, k0, g.N, khi, vecB, rb);
        }
#pragma unroll
        for (int k4 = 0; k4 < BK / 4; ++k4) {
            double a[TI], bb[TJ];
#pragma unroll
            for (int i = 0; i < TI; ++i) a[i] = lds_at<AKC, TM>(As[cur], wm + 16 * i + l16, 4 * k4 + lk);
#pragma unroll
            for (int j = 0; j < TJ; ++j) bb[j] = lds_at<BKC, BN>(Bs[cur], wn + 16 * j + l16, 4 * k4 + lk);
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], bb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            store_tile<AKC, TM>(As[cur ^ 1], ra);
            store_tile<BKC, BN>(Bs[cur ^ 1], rb);
        }
        __syncthreads();
    }

    // accumulator element v of tile (i, j): row 16 i + lane / 16 + 4 v, column 16 j + lane % 16
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = m0 + wm + 16 * i + lk + 4 * v;
            if (row >= g.M) continue;
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                const int col = n0 + wn + 16 * j + l16;
                if (col >= g.N) continue;
                double* c = C + (long long)row * g.ldc + col;
                double r = g.alpha * acc[i][j][v];
                if (g.beta != 0.0) r += g.beta * (*c);
                *c = r;
            }
        }
}

}  // namespace

int gemm_f64(tboa_ctx* ctx, const GemmF64& q) {
    if (q.M <= 0 || q.N <= 0 || q.batch <= 0) return 0;
    if (q.K < 0 || !q.A || !q.B || !q.C) return tboa_fail(ctx, TBOA_EINVAL, "gemm_f64: null operand or negative K");
    const bool akc = (q.sak == 1), bkc = (q.sbk == 1);
    if (!akc && q.sam != 1) return tboa_fail(ctx, TBOA_EINVAL, "gemm_f64: A needs a unit stride");
    if (!bkc && q.sbn != 1) return tboa_fail(ctx, TBOA_EINVAL, "gemm_f64: B needs a unit stride");
    Args a;
    a.M = q.M; a.N = q.N; a.K = q.K; a.alpha = q.alpha; a.beta = q.beta;
    a.A = q.A; a.sa_r = q.sam; a.sa_k = q.sak;
    a.B = q.B; a.sb_k = q.sbk; a.sb_r = q.sbn;
    a.C = q.C; a.ldc = q.ldc;
    a.strideA = q.strideA; a.strideB = q.strideB; a.strideC = q.strideC;
    a.strideA2 = q.strideA2; a.strideB2 = q.strideB2; a.strideC2 = q.strideC2;
    a.batch_inner = q.batch_inner > 0 ? q.batch_inner : 1;
    a.klo_m = q.klo_m; a.klo_n = q.klo_n; a.khi_m = q.khi_m; a.khi_n = q.khi_n;
    a.A2 = q.A2; a.B2 = q.A2 ? q.B2 : nullptr;
    if (q.A2 && (!q.B2 || q.klo_m || q.klo_n || q.khi_m || q.khi_n)) return tboa_fail(ctx, TBOA_EINVAL, "gemm_f64: a second operand pair needs both operands and an unrestricted contraction");
    a.skip_lower = q.skip_lower; a.skip_upper = q.skip_upper; a.skip_col0 = q.skip_col0; a.m_limit = q.m_limit; a.diag_order = q.diag_order;
    // 16-byte vector loads need every row start and the tile offsets (even) to stay 16-byte aligned
    const bool vecA = ((uintptr_t)q.A % 16 == 0) && ((uintptr_t)q.A2 % 16 == 0) && (q.strideA % 2 == 0) && (q.strideA2 % 2 == 0) && ((akc ? q.sam : q.sak) % 2 == 0);
    const bool vecB = ((uintptr_t)q.B % 16 == 0) && ((uintptr_t)q.B2 % 16 == 0) && (q.strideB % 2 == 0) && (q.strideB2 % 2 == 0) && ((bkc ? q.sbn : q.sbk) % 2 == 0);
    // algorithmic flops of a tagged launch: 2 M N K per batch entry over the contraction range each output tile really has;
    // a launch whose row count comes from device memory (m_limit) is timed but not counted
    ProfRec rec{}; bool timed = false;
    if (ctx->prof_on && q.tag >= 0) {
        double macs = 0.0;
        if (!q.m_limit)
            for (int m0 = 0; m0 < q.M; m0 += BM)
                for (int n0 = 0; n0 < q.N; n0 += BN) {
                    if (q.skip_lower && q.skip_col0 + n0 + BN <= m0) continue;
                    if (q.skip_upper && m0 + BM <= q.skip_col0 + n0) continue;
                    int klo = 0, khi = q.K;
                    if (q.klo_m) klo = std::max(klo, m0);
                    if (q.klo_n) klo = std::max(klo, n0);
                    if (q.khi_m) khi = std::min(khi, m0 + BM);
                    if (q.khi_n) khi = std::min(khi, n0 + BN);
                    if (khi > klo) macs += (double)std::min(BM, q.M - m0) * std::min(BN, q.N - n0) * (khi - klo) * (q.A2 ? 2.0 : 1.0);
                }
        TB_TRY(prof_begin(ctx, q.tag, 2.0 * macs * q.batch, rec, timed));
    }
    const bool skinny = q.M <= 32 && akc;
    dim3 grid((unsigned)cdiv64(q.N, BN), (unsigned)cdiv64(q.M, skinny ? 32 : BM), (unsigned)q.batch);
    if (grid.y > 65535 || grid.z > 65535) return tboa_fail(ctx, TBOA_EINVAL, "gemm_f64: grid too large");
    if (skinny && bkc) hipLaunchKernelGGL((gemm_f64_kernel<true, true, 32>), grid, dim3(256), 0, ctx->stream, a, vecA, vecB);
    else if (skinny) hipLaunchKernelGGL((gemm_f64_kernel<true, false, 32>), grid, dim3(256), 0, ctx->stream, a, vecA, vecB);
    else if (akc && bkc) hipLaunchKernelGGL((gemm_f64_kernel<true, true, BM>), grid, dim3(256), 0, ctx->stream, a, vecA, vecB);
    else if (akc && !bkc) hipLaunchKernelGGL((gemm_f64_kernel<true, false, BM>), grid, dim3(256), 0, ctx->stream, a, vecA, vecB);
    else if (!akc && bkc) hipLaunchKernelGGL((gemm_f64_kernel<false, true, BM>), grid, dim3(256), 0, ctx->stream, a, vecA, vecB);
    else hipLaunchKernelGGL((gemm_f64_kernel<false, false, BM>), grid, dim3(256), 0, ctx->stream, a, vecA, vecB);
    TB_KERNEL_CHECK(ctx);
    TB_TRY(prof_end(ctx, rec, timed));
    return 0;
}

extern "C" int tboa_gemm_f64(tboa_ctx* ctx, int M, int N, int K, double alpha,
                             const double* A, int64_t sam, int64_t sak, const double* B, int64_t sbk, int64_t sbn,
                             double beta, double* C, int64_t ldc,
                             int batch, int64_t strideA, int64_t strideB, int64_t strideC) {
    if (!ctx) return TBOA_EINVAL;
    GemmF64 g{};
    g.M = M; g.N = N; g.K = K; g.alpha = alpha; g.beta = beta;
    g.A = A; g.sam = sam; g.sak = sak; g.B = B; g.sbk = sbk; g.sbn = sbn;
    g.C = C; g.ldc = ldc; g.batch = batch; g.strideA = strideA; g.strideB = strideB; g.strideC = strideC;
    return gemm_f64(ctx, g);
}
