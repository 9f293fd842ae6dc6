// U = Chol(H^-1)^T (eq. 3) without forming H^-1.
//
// With V upper triangular and H = V V^T (the Cholesky factorisation taken from the last index backwards),
// H^-1 = V^-T V^-1, so U = V^-1 is upper triangular with positive diagonal and U^T U = H^-1: by uniqueness of
// the Cholesky factor it is Chol(H^-1)^T.  One blocked factorisation plus one blocked triangular inverse, all in
// fp64: diagonal blocks are factored and inverted inside LDS by one workgroup per matrix, the panel and trailing
// updates are fp64-MFMA GEMMs batched over the matrices (the per-head Hessians of W_V factor in lockstep).
#include "internal.h"

namespace {

constexpr int NB = TB_FACT_NB;

// status[0] = 1 + column of the first non-positive pivot (0 = fine), status[1] = batch index
__global__ __launch_bounds__(256) void diag_factor_kernel(double* __restrict__ H, int n, int j0, int bs,
                                                          double* __restrict__ dinv, int blk, int nblk, int* status) {
    __shared__ double V[NB][NB + 1];
    __shared__ double W[NB][NB + 1];
    const int b = blockIdx.x, t = threadIdx.x;
    double* Hb = H + (long long)b * n * n;
    for (int i = t; i < bs * bs; i += 256) {
        const int r = i / bs, c = i % bs;
        V[r][c] = (c >= r) ? Hb[(long long)(j0 + r) * n + j0 + c] : 0.0;
    }
    __syncthreads();
    // H_jj = V V^T, V upper: columns from the last to the first.  Thread (tx, ty) = (t % 64, t / 64) owns column tx of the
    // rows ty, ty + 4, ... in both phases.
    const int tx = t & 63, ty = t >> 6;
    for (int c = bs - 1; c >= 0; --c) {
        const double piv = V[c][c];
        __syncthreads();
        if (!(piv > 0.0)) {
            if (t == 0) { if (atomicCAS(&status[0], 0, 1 + j0 + c) == 0) status[1] = b; }
        }
        const double dv = (piv > 0.0) ? sqrt(piv) : 1.0;
        if (t < c) V[t][c] = V[t][c] / dv;
        if (t == c) V[c][c] = dv;
        __syncthreads();
        // trailing (upper part): V[r][r2] -= V[r][c] * V[r2][c] for r <= r2 < c
        if (tx < c) {
            const double vc = V[tx][c];
            for (int r = ty; r <= tx; r += 4) V[r][tx] -= V[r][c] * vc;
        }
        __syncthreads();
    }
    // W = V^-1 (upper), V W = I solved for all columns at once from the last row up: row r of W is final once the
    // contributions of the rows below it have been taken from the right-hand side, and is then taken from the rows above
    for (int r = ty; r < NB; r += 4) W[r][tx] = (r == tx && r < bs) ? 1.0 : 0.0;     // right-hand side, becomes W
    __syncthreads();
    for (int r = bs - 1; r >= 0; --r) {
        if (ty == 0 && tx >= r && tx < bs) W[r][tx] = W[r][tx] / V[r][r];
        __syncthreads();
        if (tx >= r && tx < bs) {
            const double wr = W[r][tx];
            for (int i = ty; i < r; i += 4) W[i][tx] -= V[i][r] * wr;
        }
        __syncthreads();
    }
    double* D = dinv + ((long long)b * nblk + blk) * NB * NB;
    for (int i = t; i < NB * NB; i += 256) {
        const int r = i / NB, c = i % NB;
        D[i] = (r < bs && c < bs) ? W[r][c] : 0.0;
    }
    for (int i = t; i < bs * bs; i += 256) {
        const int r = i / bs, c = i % bs;
        Hb[(long long)(j0 + r) * n + j0 + c] = V[r][c];   // lower part of the block becomes zero
    }
}

__global__ void clear_status_kernel(int* status) { if (threadIdx.x < 2) status[threadIdx.x] = 0; }

__global__ void place_diag_inverse_kernel(double* __restrict__ U, int n, const double* __restrict__ dinv, int nblk) {
    const int b = blockIdx.y, blk = blockIdx.x;
    const int j0 = blk * NB, bs = min(NB, n - j0);
    const double* D = dinv + ((long long)b * nblk + blk) * NB * NB;
    double* Ub = U + (long long)b * n * n;
    for (int i = threadIdx.x; i < bs * bs; i += blockDim.x) {
        const int r = i / bs, c = i % bs;
        Ub[(long long)(j0 + r) * n + j0 + c] = D[r * NB + c];
    }
}

__global__ __launch_bounds__(256) void cvt_damp_kernel(const float* __restrict__ H, double* __restrict__ out, int n, double damp) {
    __shared__ double red[256];
    const int b = blockIdx.x, t = threadIdx.x;
    const float* Hb = H + (long long)b * n * n;
    double* Ob = out + (long long)b * n * n;
    double s = 0.0;
    for (int i = t; i < n; i += 256) s += (double)Hb[(long long)i * n + i];
    red[t] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) { if (t < o) red[t] += red[t + o]; __syncthreads(); }
    const double add = damp * (red[0] / (double)n);
    for (int i = t; i < n; i += 256) Ob[(long long)i * n + i] = (double)Hb[(long long)i * n + i] + add;
}

__global__ void cvt_offdiag_kernel(const float* __restrict__ H, double* __restrict__ out, int n, long long total) {
    const long long nn = (long long)n * n;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const long long e = i % nn;
        const int r = (int)(e / n), c = (int)(e % n);
        if (r != c) out[i] = (double)H[i];
    }
}

}  // namespace

int launch_f32_to_f64_damp(tboa_ctx* ctx, int n, int batch, const float* H, double damp, double* out) {
    const long long total = (long long)batch * n * n;
    long long g = (total + 255) / 256; if (g > 16384) g = 16384;
    hipLaunchKernelGGL(cvt_offdiag_kernel, dim3((unsigned)g), dim3(256), 0, ctx->stream, H, out, n, total);
    hipLaunchKernelGGL(cvt_damp_kernel, dim3(batch), dim3(256), 0, ctx->stream, H, out, n, damp);
    TB_KERNEL_CHECK(ctx);
    return 0;
}

// Two levels of blocking.  Diagonal blocks of NB columns are factored (and inverted) in LDS; an outer block of OB columns
// is finished block by block with updates confined to its own columns, after which ONE update with an OB-deep
// contraction carries it into the rest of the matrix: the large updates are bound by the matrix cores, not by reading
// and writing the trailing matrix once per NB columns.  The inverse is assembled the same way, OB columns at a time.
int chol_status_f64(tboa_ctx* ctx, int status_slot) {
    TB_HIP(ctx, hipMemcpyAsync(ctx->h_status + status_slot, ctx->d_status + status_slot, 2 * sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    TB_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->h_status[status_slot] != 0)
        return tboa_fail(ctx, TBOA_ENOTSPD, "Hessian %d of the batch is not positive definite: pivot %d is not positive",
                         ctx->h_status[status_slot + 1], ctx->h_status[status_slot] - 1);
    return 0;
}

int chol_inv_upper_f64(tboa_ctx* ctx, int n, int batch, double* H, double* U, double* tmp, double* dinv, int status_slot, bool defer_status) {
    int* status = ctx->d_status + status_slot;
    constexpr int OB = TB_FACT_OB, IPB = OB / NB;
    const int nblk = (n + NB - 1) / NB, nob = (n + OB - 1) / OB;
    const int TL = chol_tmp_pitch(n);     // row pitch of tmp: a matrix of one outer block only ever holds NB columns there
    const long long nn = (long long)n * n, dstride = (long long)nblk * NB * NB;
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(64), 0, ctx->stream, status);
    TB_KERNEL_CHECK(ctx);
    // ---- H = V V^T from the last column to the first
    for (int ob = nob - 1; ob >= 0; --ob) {
        const int J0 = ob * OB, J1 = (J0 + OB < n) ? J0 + OB : n;
        const int blk_hi = (J1 + NB - 1) / NB - 1, blk_lo = ob * IPB;
        for (int blk = blk_hi; blk >= blk_lo; --blk) {
            const int j0 = blk * NB, bs = (n - j0 < NB) ? n - j0 : NB;
            hipLaunchKernelGGL(diag_factor_kernel, dim3(batch), dim3(256), 0, ctx->stream, H, n, j0, bs, dinv, blk, nblk, status);
            TB_KERNEL_CHECK(ctx);
            if (j0 == 0) break;
            // panel: V[0:j0, blk] = H[0:j0, blk] Vinv_jj^T   (in place: one column tile, each workgroup owns its rows)
            GemmF64 p{};
            p.M = j0; p.N = bs; p.K = bs; p.alpha = 1.0; p.beta = 0.0;
            p.A = H + j0; p.sam = n; p.sak = 1;
            p.B = dinv + (long long)blk * NB * NB; p.sbk = 1; p.sbn = NB;
            p.C = H + j0; p.ldc = n;
            p.batch = batch; p.strideA = nn; p.strideB = dstride; p.strideC = nn;
            TB_TRY(gemm_f64(ctx, p));
            if (j0 > J0) {   // inside the outer block: H[0:j0, J0:j0] -= V[0:j0, blk] V[J0:j0, blk]^T  (upper part)
                GemmF64 s{};
                s.M = j0; s.N = j0 - J0; s.K = bs; s.alpha = -1.0; s.beta = 1.0;
                s.A = H + j0; s.sam = n; s.sak = 1;
                s.B = H + (long long)J0 * n + j0; s.sbk = 1; s.sbn = n;
                s.C = H + J0; s.ldc = n; s.skip_lower = 1; s.skip_col0 = J0;
                s.batch = batch; s.strideA = nn; s.strideB = nn; s.strideC = nn;
                TB_TRY(gemm_f64(ctx, s));
            }
        }
        if (J0 > 0) {   // H[0:J0, 0:J0] -= V[0:J0, ob] V[0:J0, ob]^T  (upper part)
            GemmF64 s{};
            s.M = J0; s.N = J0; s.K = J1 - J0; s.alpha = -1.0; s.beta = 1.0;
            s.A = H + J0; s.sam = n; s.sak = 1;
            s.B = H + J0; s.sbk = 1; s.sbn = n;
            s.C = H; s.ldc = n; s.skip_lower = 1;
            s.batch = batch; s.strideA = nn; s.strideB = nn; s.strideC = nn;
            TB_TRY(gemm_f64(ctx, s));
        }
    }
    // ---- U = V^-1
    TB_TRY(launch_fill_f64(ctx, U, (int64_t)batch * nn, 0.0));
    hipLaunchKernelGGL(place_diag_inverse_kernel, dim3(nblk, batch), dim3(256), 0, ctx->stream, U, n, dinv, nblk);
    TB_KERNEL_CHECK(ctx);
    for (int ob = 0; ob < nob; ++ob) {
        const int J0 = ob * OB, J1 = (J0 + OB < n) ? J0 + OB : n;
        const int blk_hi = (J1 + NB - 1) / NB - 1, blk_lo = ob * IPB;
        for (int blk = blk_lo + 1; blk <= blk_hi; ++blk) {   // the diagonal block of the outer block: U[J0:j0, blk]
            const int j0 = blk * NB, bs = (n - j0 < NB) ? n - j0 : NB, m = j0 - J0;
            GemmF64 a{};   // tmp = U[J0:j0, J0:j0] V[J0:j0, blk]
            a.M = m; a.N = bs; a.K = m; a.alpha = 1.0; a.beta = 0.0;
            a.A = U + (long long)J0 * n + J0; a.sam = n; a.sak = 1; a.klo_m = 1;
            a.B = H + (long long)J0 * n + j0; a.sbk = n; a.sbn = 1;
            a.C = tmp; a.ldc = TL;
            a.batch = batch; a.strideA = nn; a.strideB = nn; a.strideC = (long long)n * TL;
            TB_TRY(gemm_f64(ctx, a));
            GemmF64 c{};   // U[J0:j0, blk] = -tmp Vinv_jj
            c.M = m; c.N = bs; c.K = bs; c.alpha = -1.0; c.beta = 0.0;
            c.A = tmp; c.sam = TL; c.sak = 1;
            c.B = dinv + (long long)blk * NB * NB; c.sbk = NB; c.sbn = 1;
            c.C = U + (long long)J0 * n + j0; c.ldc = n;
            c.batch = batch; c.strideA = (long long)n * TL; c.strideB = dstride; c.strideC = nn;
            TB_TRY(gemm_f64(ctx, c));
        }
        if (J0 > 0) {
            const int w = J1 - J0;
            GemmF64 a{};   // tmp = U[0:J0, 0:J0] V[0:J0, ob]
            a.M = J0; a.N = w; a.K = J0; a.alpha = 1.0; a.beta = 0.0;
            a.A = U; a.sam = n; a.sak = 1; a.klo_m = 1;
            a.B = H + J0; a.sbk = n; a.sbn = 1;
            a.C = tmp; a.ldc = TL;
            a.batch = batch; a.strideA = nn; a.strideB = nn; a.strideC = (long long)n * TL;
            TB_TRY(gemm_f64(ctx, a));
            GemmF64 c{};   // U[0:J0, ob] = -tmp U[ob, ob]   (U[ob, ob] upper: k <= column)
            c.M = J0; c.N = w; c.K = w; c.alpha = -1.0; c.beta = 0.0;
            c.A = tmp; c.sam = TL; c.sak = 1;
            c.B = U + (long long)J0 * n + J0; c.sbk = n; c.sbn = 1; c.khi_n = 1;
            c.C = U + J0; c.ldc = n;
            c.batch = batch; c.strideA = (long long)n * TL; c.strideB = nn; c.strideC = nn;
            TB_TRY(gemm_f64(ctx, c));
        }
    }
    return defer_status ? 0 : chol_status_f64(ctx, status_slot);
}

extern "C" int tboa_chol_inv_upper(tboa_ctx* ctx, int n, int batch, const float* H, double damp, double* U) {
    if (!ctx) return TBOA_EINVAL;
    if (n <= 0 || batch <= 0 || !H || !U) return tboa_fail(ctx, TBOA_EINVAL, "chol_inv_upper: bad arguments");
    const int nblk = (n + NB - 1) / NB;
    Arena plan(nullptr);
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        double* H64 = ar.get<double>((size_t)batch * n * n);
        double* tmp = ar.get<double>((size_t)batch * n * chol_tmp_pitch(n));
        double* dinv = ar.get<double>((size_t)batch * nblk * NB * NB);
        if (!pass) { TB_TRY(tboa_ws_reserve(ctx, ar.off)); continue; }
        TB_TRY(launch_f32_to_f64_damp(ctx, n, batch, H, damp, H64));
        TB_TRY(chol_inv_upper_f64(ctx, n, batch, H64, U, tmp, dinv));
    }
    return 0;
}

// ------------------------------------------------------------------------------------------------
// The same factorisation for callers that cannot allocate: its three temporaries (the fp64 copy of H that becomes V,
// the panel buffer of the triangular inverse, the inverted diagonal blocks) live in a file-scope device array instead
// of the context's workspace.  Every GPU the library runs on holds its own copy of the array until the process ends;
// its address on a device is looked up once, by tboa_create with that device current.  All calls on one GPU share the
// array: two calls that overlap in time on the same GPU (different streams, different host threads) race.
namespace {
constexpr size_t STATIC_REGION = (size_t)1 << 20;                    // doubles per temporary: 8 MiB
__device__ __align__(256) double scratch[3 * STATIC_REGION];         // 24 MiB
constexpr int MAX_DEVICES = 64;
double* scratch_on_device[MAX_DEVICES];                              // device address of `scratch`, per device (0 = not looked up)
}  // namespace

int chol_static_init(int device) {
    if (device < 0 || device >= MAX_DEVICES) return TBOA_EINVAL;
    if (scratch_on_device[device]) return 0;
    double* p = nullptr;
    if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return TBOA_EHIP; }
    scratch_on_device[device] = p;
    return 0;
}

extern "C" size_t tboa_chol_inv_upper_static_max_elems(void) { return STATIC_REGION; }

extern "C" int tboa_chol_inv_upper_static(tboa_ctx* ctx, int n, int batch, const float* H, double damp, double* U) {
    if (!ctx) return TBOA_EINVAL;
    if (n <= 0 || batch <= 0 || !H || !U) return tboa_fail(ctx, TBOA_EINVAL, "chol_inv_upper_static: bad arguments");
    const size_t n64 = (size_t)((n + NB - 1) / NB) * NB;
    if (n > TB_FACT_OB || (size_t)batch * n64 * n64 > STATIC_REGION)
        return tboa_fail(ctx, TBOA_EINVAL, "chol_inv_upper_static: n = %d, batch = %d exceed the static scratch (n <= %d and "
                         "batch * roundup64(n)^2 <= %zu); use tboa_chol_inv_upper", n, batch, TB_FACT_OB, STATIC_REGION);
    double* base = (ctx->device >= 0 && ctx->device < MAX_DEVICES) ? scratch_on_device[ctx->device] : nullptr;
    if (!base) return tboa_fail(ctx, TBOA_EHIP, "chol_inv_upper_static: the static scratch of device %d was not found at tboa_create", ctx->device);
    // H64: batch n^2; tmp: batch n 64 (one outer block: chol_tmp_pitch(n) = 64); dinv: batch ceil(n / 64) 64^2 -- each within a region
    double* H64 = base; double* tmp = base + STATIC_REGION; double* dinv = base + 2 * STATIC_REGION;
    TB_TRY(launch_f32_to_f64_damp(ctx, n, batch, H, damp, H64));
    return chol_inv_upper_f64(ctx, n, batch, H64, U, tmp, dinv);
}
