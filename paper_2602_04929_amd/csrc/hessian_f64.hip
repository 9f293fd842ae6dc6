// Table 1 Hessians for fp32 inputs: every contraction on the fp64 matrix cores (small problems, reference-grade
// accuracy).  Literal order of Table 1: projections, A_h = softmax(Q_h K_h^T / sqrt(d_h)) per sequence and head,
// Y = A_h X_s, sums of outer products over tokens.  The bf16 path for large blocks lives in hessian_bf16.hip.
#include "internal.h"
#include <math.h>

namespace {

// P[t, :] = softmax(S[t, :k_end]) with k_end = t+1 (causal) or L; zeros elsewhere.  One wavefront per row.
__global__ __launch_bounds__(256) void softmax_f64_kernel(const double* __restrict__ S, double* __restrict__ P, int L, int causal) {
    const int lane = threadIdx.x & 63, t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= L) return;
    const double* s = S + (long long)t * L; double* p = P + (long long)t * L;
    const int kend = causal ? t + 1 : L;
    double m = -INFINITY;
    for (int k = lane; k < kend; k += 64) m = fmax(m, s[k]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmax(m, __shfl_xor(m, o, 64));
    double sum = 0.0;
    for (int k = lane; k < kend; k += 64) sum += exp(s[k] - m);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    for (int k = lane; k < L; k += 64) p[k] = (k < kend) ? exp(s[k] - m) / sum : 0.0;
}

struct F64Attn {
    tboa_ctx* ctx; const tboa_attn_desc* d;
    int T, dm, Hq, Hkv, dh, L, S, rep, dq, dkv;
};

inline GemmF64 mk(int M, int N, int K, double alpha, const double* A, int64_t sam, int64_t sak, const double* B, int64_t sbk,
                  int64_t sbn, double beta, double* C, int64_t ldc) {
    GemmF64 g{};
    g.M = M; g.N = N; g.K = K; g.alpha = alpha; g.beta = beta; g.A = A; g.sam = sam; g.sak = sak; g.B = B; g.sbk = sbk; g.sbn = sbn;
    g.C = C; g.ldc = ldc; g.batch = 1;
    return g;
}

// probabilities of (sequence s, query head h) from the projected activations Qa [T, dq], Ka [T, dkv]
int attn_probs(const F64Attn& a, const double* Qa, const double* Ka, int s, int h, double* Sbuf, double* Pbuf) {
    const int g = h / a.rep, L = a.L;
    TB_TRY(gemm_f64(a.ctx, mk(L, L, a.dh, 1.0 / sqrt((double)a.dh), Qa + (long long)s * L * a.dq + h * a.dh, a.dq, 1,
                              Ka + (long long)s * L * a.dkv + g * a.dh, 1, a.dkv, 0.0, Sbuf, L)));
    hipLaunchKernelGGL(softmax_f64_kernel, dim3((L + 3) / 4), dim3(256), 0, a.ctx->stream, Sbuf, Pbuf, L, a.d->causal);
    TB_HIP(a.ctx, hipGetLastError());
    return 0;
}

}  // namespace

int build_hessians_f64(tboa_ctx* ctx, const tboa_attn_desc* d, const void* X, const void* X_fp, const void* Wq, const void* Wk,
                       const void* Wv, const void* Wo, float* Hin_qk, float* R_qk, float* Hout_q, float* Hout_k, float* Hin_v,
                       float* R_v, float* Hout_v) {
    (void)Wv;
    F64Attn a{ctx, d, d->n_seqs * d->seq_len, d->d_model, d->n_q_heads, d->n_kv_heads, d->head_dim, d->seq_len, d->n_seqs,
              d->n_q_heads / d->n_kv_heads, d->n_q_heads * d->head_dim, d->n_kv_heads * d->head_dim};
    const int T = a.T, dm = a.dm, Hq = a.Hq, Hkv = a.Hkv, dh = a.dh, L = a.L, dq = a.dq, dkv = a.dkv;
    const bool fp = X_fp != nullptr;
    const bool rv = fp && R_v;
    double *X64, *Xf64, *dX, *Wq64, *Wk64, *Wo64, *Qa, *Ka, *Qf, *Kf, *Sb, *Pb, *Y, *Yf, *Hin, *Rq, *Hoq, *Hok, *Hiv, *Rv, *Hov;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        X64 = ar.get<double>((size_t)T * dm); Xf64 = fp ? ar.get<double>((size_t)T * dm) : nullptr; dX = fp ? ar.get<double>((size_t)T * dm) : nullptr;
        Wq64 = ar.get<double>((size_t)dq * dm); Wk64 = ar.get<double>((size_t)dkv * dm); Wo64 = ar.get<double>((size_t)dm * dq);
        Qa = ar.get<double>((size_t)T * dq); Ka = ar.get<double>((size_t)T * dkv);
        Qf = rv ? ar.get<double>((size_t)T * dq) : nullptr; Kf = rv ? ar.get<double>((size_t)T * dkv) : nullptr;
        Sb = ar.get<double>((size_t)L * L); Pb = ar.get<double>((size_t)L * L);
        Y = ar.get<double>((size_t)L * dm); Yf = rv ? ar.get<double>((size_t)L * dm) : nullptr;
        Hin = ar.get<double>((size_t)dm * dm); Rq = fp ? ar.get<double>((size_t)dm * dm) : nullptr;
        Hoq = ar.get<double>((size_t)Hq * dh * dh); Hok = ar.get<double>((size_t)Hkv * dh * dh); Hov = ar.get<double>((size_t)Hkv * dh * dh);
        Hiv = ar.get<double>((size_t)Hkv * dm * dm); Rv = rv ? ar.get<double>((size_t)Hkv * dm * dm) : nullptr;
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    TB_TRY(launch_cvt_to_f64(ctx, X, TBOA_F32, X64, (int64_t)T * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wq, TBOA_F32, Wq64, (int64_t)dq * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wk, TBOA_F32, Wk64, (int64_t)dkv * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wo, TBOA_F32, Wo64, (int64_t)dm * dq));
    // H_in = X X^T (paper's X is channels x tokens) and R = alpha dX X^T
    TB_TRY(gemm_f64(ctx, mk(dm, dm, T, 1.0, X64, 1, dm, X64, dm, 1, 0.0, Hin, dm)));
    if (fp) {
        TB_TRY(launch_cvt_to_f64(ctx, X_fp, TBOA_F32, Xf64, (int64_t)T * dm));
        TB_TRY(launch_sub_f64(ctx, X64, Xf64, dX, (int64_t)T * dm));
        TB_TRY(gemm_f64(ctx, mk(dm, dm, T, d->alpha, dX, 1, dm, X64, dm, 1, 0.0, Rq, dm)));
    }
    // projections
    TB_TRY(gemm_f64(ctx, mk(T, dq, dm, 1.0, X64, dm, 1, Wq64, 1, dm, 0.0, Qa, dq)));
    TB_TRY(gemm_f64(ctx, mk(T, dkv, dm, 1.0, X64, dm, 1, Wk64, 1, dm, 0.0, Ka, dkv)));
    if (rv) {
        TB_TRY(gemm_f64(ctx, mk(T, dq, dm, 1.0, Xf64, dm, 1, Wq64, 1, dm, 0.0, Qf, dq)));
        TB_TRY(gemm_f64(ctx, mk(T, dkv, dm, 1.0, Xf64, dm, 1, Wk64, 1, dm, 0.0, Kf, dkv)));
    }
    // H_out of W_Q,h: K_g^T K_g ; of W_K,g: sum_h Q_h^T Q_h ; of W_V,g: sum_h W_out,h^T W_out,h
    TB_TRY(launch_fill_f64(ctx, Hok, (int64_t)Hkv * dh * dh, 0.0));
    TB_TRY(launch_fill_f64(ctx, Hov, (int64_t)Hkv * dh * dh, 0.0));
    for (int h = 0; h < Hq; ++h) {
        const int g = h / a.rep;
        TB_TRY(gemm_f64(ctx, mk(dh, dh, T, 1.0, Ka + g * dh, 1, dkv, Ka + g * dh, dkv, 1, 0.0, Hoq + (long long)h * dh * dh, dh)));
        TB_TRY(gemm_f64(ctx, mk(dh, dh, T, 1.0, Qa + h * dh, 1, dq, Qa + h * dh, dq, 1, 1.0, Hok + (long long)g * dh * dh, dh)));
        TB_TRY(gemm_f64(ctx, mk(dh, dh, dm, 1.0, Wo64 + h * dh, 1, dq, Wo64 + h * dh, dq, 1, 1.0, Hov + (long long)g * dh * dh, dh)));
    }
    // H_in of W_V,g: sum over heads of the group and sequences of (A_h X_s)^T (A_h X_s)
    TB_TRY(launch_fill_f64(ctx, Hiv, (int64_t)Hkv * dm * dm, 0.0));
    if (rv) TB_TRY(launch_fill_f64(ctx, Rv, (int64_t)Hkv * dm * dm, 0.0));
    for (int s = 0; s < a.S; ++s)
        for (int h = 0; h < Hq; ++h) {
            const int g = h / a.rep;
            const double* Xs = X64 + (long long)s * L * dm;
            TB_TRY(attn_probs(a, Qa, Ka, s, h, Sb, Pb));
            TB_TRY(gemm_f64(ctx, mk(L, dm, L, 1.0, Pb, L, 1, Xs, dm, 1, 0.0, Y, dm)));
            TB_TRY(gemm_f64(ctx, mk(dm, dm, L, 1.0, Y, 1, dm, Y, dm, 1, 1.0, Hiv + (long long)g * dm * dm, dm)));
            if (rv) {
                TB_TRY(attn_probs(a, Qf, Kf, s, h, Sb, Pb));
                TB_TRY(gemm_f64(ctx, mk(L, dm, L, 1.0, Pb, L, 1, Xf64 + (long long)s * L * dm, dm, 1, 0.0, Yf, dm)));
                TB_TRY(launch_sub_f64(ctx, Y, Yf, Yf, (int64_t)L * dm));
                TB_TRY(gemm_f64(ctx, mk(dm, dm, L, d->alpha, Yf, 1, dm, Y, dm, 1, 1.0, Rv + (long long)g * dm * dm, dm)));
            }
        }
    if (Hin_qk) TB_TRY(launch_cvt_f64_to_f32(ctx, Hin, Hin_qk, (int64_t)dm * dm));
    if (fp && R_qk) TB_TRY(launch_cvt_f64_to_f32(ctx, Rq, R_qk, (int64_t)dm * dm));
    if (Hout_q) TB_TRY(launch_cvt_f64_to_f32(ctx, Hoq, Hout_q, (int64_t)Hq * dh * dh));
    if (Hout_k) TB_TRY(launch_cvt_f64_to_f32(ctx, Hok, Hout_k, (int64_t)Hkv * dh * dh));
    if (Hout_v) TB_TRY(launch_cvt_f64_to_f32(ctx, Hov, Hout_v, (int64_t)Hkv * dh * dh));
    if (Hin_v) TB_TRY(launch_cvt_f64_to_f32(ctx, Hiv, Hin_v, (int64_t)Hkv * dm * dm));
    if (rv) TB_TRY(launch_cvt_f64_to_f32(ctx, Rv, R_v, (int64_t)Hkv * dm * dm));
    return 0;
}

// attention output concat_h(A_h V_g(h)) [T, dq] for weights Wq/Wk/Wv (fp64) on activations Xa (fp64)
static int attn_output_f64(const F64Attn& a, const double* Xa, const double* Wq64, const double* Wk64, const double* Wv64,
                           double* Qa, double* Ka, double* Va, double* Sb, double* Pb, double* O) {
    tboa_ctx* ctx = a.ctx;
    const int T = a.T, dm = a.dm, dq = a.dq, dkv = a.dkv, L = a.L, dh = a.dh;
    TB_TRY(gemm_f64(ctx, mk(T, dq, dm, 1.0, Xa, dm, 1, Wq64, 1, dm, 0.0, Qa, dq)));
    TB_TRY(gemm_f64(ctx, mk(T, dkv, dm, 1.0, Xa, dm, 1, Wk64, 1, dm, 0.0, Ka, dkv)));
    TB_TRY(gemm_f64(ctx, mk(T, dkv, dm, 1.0, Xa, dm, 1, Wv64, 1, dm, 0.0, Va, dkv)));
    for (int s = 0; s < a.S; ++s)
        for (int h = 0; h < a.Hq; ++h) {
            const int g = h / a.rep;
            TB_TRY(attn_probs(a, Qa, Ka, s, h, Sb, Pb));
            TB_TRY(gemm_f64(ctx, mk(L, dh, L, 1.0, Pb, L, 1, Va + (long long)s * L * dkv + g * dh, dkv, 1, 0.0,
                                    O + (long long)s * L * dq + h * dh, dq)));
        }
    return 0;
}

int build_hessian_out_proj_f64(tboa_ctx* ctx, const tboa_attn_desc* d, const void* X, const void* X_fp, const float* Wq_deq,
                               const float* Wk_deq, const float* Wv_deq, const void* Wq, const void* Wk, const void* Wv,
                               float* Hin_o, float* R_o) {
    F64Attn a{ctx, d, d->n_seqs * d->seq_len, d->d_model, d->n_q_heads, d->n_kv_heads, d->head_dim, d->seq_len, d->n_seqs,
              d->n_q_heads / d->n_kv_heads, d->n_q_heads * d->head_dim, d->n_kv_heads * d->head_dim};
    const int T = a.T, dm = a.dm, L = a.L, dq = a.dq, dkv = a.dkv;
    const bool fp = X_fp && R_o;
    double *X64, *Wq64, *Wk64, *Wv64, *Qa, *Ka, *Va, *Sb, *Pb, *O, *Of, *H;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        X64 = ar.get<double>((size_t)T * dm);
        Wq64 = ar.get<double>((size_t)dq * dm); Wk64 = ar.get<double>((size_t)dkv * dm); Wv64 = ar.get<double>((size_t)dkv * dm);
        Qa = ar.get<double>((size_t)T * dq); Ka = ar.get<double>((size_t)T * dkv); Va = ar.get<double>((size_t)T * dkv);
        Sb = ar.get<double>((size_t)L * L); Pb = ar.get<double>((size_t)L * L);
        O = ar.get<double>((size_t)T * dq); Of = fp ? ar.get<double>((size_t)T * dq) : nullptr;
        H = ar.get<double>((size_t)dq * dq);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    TB_TRY(launch_cvt_to_f64(ctx, X, TBOA_F32, X64, (int64_t)T * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wq_deq, TBOA_F32, Wq64, (int64_t)dq * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wk_deq, TBOA_F32, Wk64, (int64_t)dkv * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wv_deq, TBOA_F32, Wv64, (int64_t)dkv * dm));
    TB_TRY(attn_output_f64(a, X64, Wq64, Wk64, Wv64, Qa, Ka, Va, Sb, Pb, O));
    TB_TRY(gemm_f64(ctx, mk(dq, dq, T, 1.0, O, 1, dq, O, dq, 1, 0.0, H, dq)));
    TB_TRY(launch_cvt_f64_to_f32(ctx, H, Hin_o, (int64_t)dq * dq));
    if (fp) {
        TB_TRY(launch_cvt_to_f64(ctx, X_fp, TBOA_F32, X64, (int64_t)T * dm));
        TB_TRY(launch_cvt_to_f64(ctx, Wq, TBOA_F32, Wq64, (int64_t)dq * dm));
        TB_TRY(launch_cvt_to_f64(ctx, Wk, TBOA_F32, Wk64, (int64_t)dkv * dm));
        TB_TRY(launch_cvt_to_f64(ctx, Wv, TBOA_F32, Wv64, (int64_t)dkv * dm));
        TB_TRY(attn_output_f64(a, X64, Wq64, Wk64, Wv64, Qa, Ka, Va, Sb, Pb, Of));
        TB_TRY(launch_sub_f64(ctx, O, Of, Of, (int64_t)T * dq));
        TB_TRY(gemm_f64(ctx, mk(dq, dq, T, d->alpha, Of, 1, dq, O, dq, 1, 0.0, H, dq)));
        TB_TRY(launch_cvt_f64_to_f32(ctx, H, R_o, (int64_t)dq * dq));
    }
    return 0;
}

// attention output concat_h(A_h V_g(h)) [T, Hq dh] (fp32) of fp32 activations and weights, on the fp64 matrix cores
int attention_forward_f64(tboa_ctx* ctx, const tboa_attn_desc* d, const float* X, const float* Wq, const float* Wk, const float* Wv, float* O) {
    F64Attn a{ctx, d, d->n_seqs * d->seq_len, d->d_model, d->n_q_heads, d->n_kv_heads, d->head_dim, d->seq_len, d->n_seqs,
              d->n_q_heads / d->n_kv_heads, d->n_q_heads * d->head_dim, d->n_kv_heads * d->head_dim};
    const int T = a.T, dm = a.dm, L = a.L, dq = a.dq, dkv = a.dkv;
    double *X64, *Wq64, *Wk64, *Wv64, *Qa, *Ka, *Va, *Sb, *Pb, *O64;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        X64 = ar.get<double>((size_t)T * dm);
        Wq64 = ar.get<double>((size_t)dq * dm); Wk64 = ar.get<double>((size_t)dkv * dm); Wv64 = ar.get<double>((size_t)dkv * dm);
        Qa = ar.get<double>((size_t)T * dq); Ka = ar.get<double>((size_t)T * dkv); Va = ar.get<double>((size_t)T * dkv);
        Sb = ar.get<double>((size_t)L * L); Pb = ar.get<double>((size_t)L * L);
        O64 = ar.get<double>((size_t)T * dq);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    TB_TRY(launch_cvt_to_f64(ctx, X, TBOA_F32, X64, (int64_t)T * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wq, TBOA_F32, Wq64, (int64_t)dq * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wk, TBOA_F32, Wk64, (int64_t)dkv * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wv, TBOA_F32, Wv64, (int64_t)dkv * dm));
    TB_TRY(attn_output_f64(a, X64, Wq64, Wk64, Wv64, Qa, Ka, Va, Sb, Pb, O64));
    return launch_cvt_f64_to_f32(ctx, O64, O, (int64_t)T * dq);
}

namespace {
__global__ void add_cvt_kernel(const double* __restrict__ Y, const float* __restrict__ Res, float* __restrict__ out, long long n) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
        out[i] = (float)(Res ? Y[i] + (double)Res[i] : Y[i]);
}
}  // namespace

// Y = X W^T (+ Res), fp32 in and out, on the fp64 matrix cores
int linear_forward_f64(tboa_ctx* ctx, long long T, int din, int dout, const float* X, const float* W, const float* Res, float* Y) {
    double *X64, *W64, *Y64;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        X64 = ar.get<double>((size_t)T * din); W64 = ar.get<double>((size_t)dout * din); Y64 = ar.get<double>((size_t)T * dout);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    TB_TRY(launch_cvt_to_f64(ctx, X, TBOA_F32, X64, (int64_t)T * din));
    TB_TRY(launch_cvt_to_f64(ctx, W, TBOA_F32, W64, (int64_t)dout * din));
    TB_TRY(gemm_f64(ctx, mk((int)T, dout, din, 1.0, X64, din, 1, W64, 1, din, 0.0, Y64, dout)));
    long long n = T * dout, gb = (n + 255) / 256; if (gb > 16384) gb = 16384;
    hipLaunchKernelGGL(add_cvt_kernel, dim3((unsigned)gb), dim3(256), 0, ctx->stream, Y64, Res, Y, n);
    TB_HIP(ctx, hipGetLastError());
    return 0;
}

namespace {
__global__ void swiglu_f64_kernel(const double* __restrict__ G, const double* __restrict__ U, float* __restrict__ out, long long n) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
        const double g = G[i];
        out[i] = (float)((g / (1.0 + exp(-g))) * U[i]);
    }
}
}  // namespace

// fp32 inputs: H = X^T X and R = alpha (X - X~)^T X on the fp64 matrix cores
int build_hessian_linear_f64(tboa_ctx* ctx, long long T, int n, double alpha, const float* X, const float* X_fp, float* H_in, float* R) {
    const bool fp = X_fp && R;
    double *X64, *Xf64, *H64;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        X64 = ar.get<double>((size_t)T * n); Xf64 = fp ? ar.get<double>((size_t)T * n) : nullptr; H64 = ar.get<double>((size_t)n * n);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    TB_TRY(launch_cvt_to_f64(ctx, X, TBOA_F32, X64, (int64_t)T * n));
    TB_TRY(gemm_f64(ctx, mk(n, n, (int)T, 1.0, X64, 1, n, X64, n, 1, 0.0, H64, n)));
    TB_TRY(launch_cvt_f64_to_f32(ctx, H64, H_in, (int64_t)n * n));
    if (fp) {
        TB_TRY(launch_cvt_to_f64(ctx, X_fp, TBOA_F32, Xf64, (int64_t)T * n));
        TB_TRY(launch_sub_f64(ctx, X64, Xf64, Xf64, (int64_t)T * n));
        TB_TRY(gemm_f64(ctx, mk(n, n, (int)T, alpha, Xf64, 1, n, X64, n, 1, 0.0, H64, n)));
        TB_TRY(launch_cvt_f64_to_f32(ctx, H64, R, (int64_t)n * n));
    }
    return 0;
}

int swiglu_forward_f64(tboa_ctx* ctx, long long T, int d, int dff, const float* X, const float* Wg, const float* Wu, float* Act) {
    double *X64, *Wg64, *Wu64, *G, *U;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        X64 = ar.get<double>((size_t)T * d); Wg64 = ar.get<double>((size_t)dff * d); Wu64 = ar.get<double>((size_t)dff * d);
        G = ar.get<double>((size_t)T * dff); U = ar.get<double>((size_t)T * dff);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    TB_TRY(launch_cvt_to_f64(ctx, X, TBOA_F32, X64, (int64_t)T * d));
    TB_TRY(launch_cvt_to_f64(ctx, Wg, TBOA_F32, Wg64, (int64_t)dff * d));
    TB_TRY(launch_cvt_to_f64(ctx, Wu, TBOA_F32, Wu64, (int64_t)dff * d));
    TB_TRY(gemm_f64(ctx, mk((int)T, dff, d, 1.0, X64, d, 1, Wg64, 1, d, 0.0, G, dff)));
    TB_TRY(gemm_f64(ctx, mk((int)T, dff, d, 1.0, X64, d, 1, Wu64, 1, d, 0.0, U, dff)));
    long long n = T * dff, gb = (n + 255) / 256; if (gb > 16384) gb = 16384;
    hipLaunchKernelGGL(swiglu_f64_kernel, dim3((unsigned)gb), dim3(256), 0, ctx->stream, G, U, Act, n);
    TB_HIP(ctx, hipGetLastError());
    return 0;
}
