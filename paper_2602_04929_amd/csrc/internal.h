// Internal declarations shared by the translation units of libturboboa (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include <string.h>
#include <vector>
#include "../../include/turboboa.h"

struct ProfRec { hipEvent_t a, b; int tag; double flops; };

struct TileOrder { int tiles_m, tiles_n, flags; int* dev; int count; };   // gemm_bf16: launch order of the output tiles
// gemm_bf16, persistent kernel: per workgroup the list of (batch entry, tm << 16 | tn) it works through, `rounds` entries each
struct TileSchedule { int tiles_m, tiles_n, flags, batch, seg_len; int2* dev; int rounds, wgs; };

struct tboa_ctx {
    int device;
    hipStream_t stream;
    char err[768];
    void* ws;            // context-owned workspace
    size_t ws_bytes;
    int* d_status;       // device status words: [0..3] factorisation breakdown (two slots), [4] integer-form check,
                         // [TB_GSTAT_WORD ..] bookkeeping of the two-phase grid search
    int* h_status;       // pinned host mirror
    hipStream_t aux;     // second stream (default priority) for work of one call that is independent of what `stream` does
    hipEvent_t ev_fork, ev_join;
    int prof_on;         // record HIP events around tagged GEMM launches
    std::vector<ProfRec> prof;
    long long counters[8];   // tboa_counter_id
    int plan_only = 0;       // a host-only context of the workspace queries: tboa_ws_reserve records the request and stops the call
    size_t plan_bytes = 0;
    std::vector<TileOrder> tile_orders;   // device tables owned by the context
    std::vector<TileSchedule> tile_schedules;
};

#define TB_GSTAT_WORD 8
int tboa_fail(tboa_ctx* ctx, int code, const char* fmt, ...);

#define TB_HIP(ctx, call)                                                                          \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess)                                                                      \
            return tboa_fail(ctx, TBOA_EHIP, "%s:%d %s: %s", __FILE__, __LINE__, #call,            \
                             hipGetErrorString(e_));                                               \
    } while (0)

#define TB_TRY(expr)                                                                               \
    do {                                                                                           \
        int rc_ = (expr);                                                                          \
        if (rc_ != 0) return rc_;                                                                  \
    } while (0)

#define TB_KERNEL_CHECK(ctx) TB_HIP(ctx, hipGetLastError())

// Bump allocator over the context workspace.  With base == nullptr it only counts bytes, so the same
// planning code sizes the workspace and then carves it.
struct Arena {
    char* base;
    size_t off;
    explicit Arena(void* b) : base((char*)b), off(0) {}
    template <typename T>
    T* get(size_t n) {
        size_t bytes = (n * sizeof(T) + 255) & ~(size_t)255;
        T* p = base ? (T*)(base + off) : nullptr;
        off += bytes;
        return p;
    }
};
// returns TB_PLAN_STOP (not an error) on a plan-only context, after recording `bytes`
#define TB_PLAN_STOP 1000
int tboa_ws_reserve(tboa_ctx* ctx, size_t bytes);

static inline int64_t cdiv64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------- gemm_f64.hip
struct GemmF64 {
    int M, N, K;
    double alpha, beta;
    const double* A; int64_t sam, sak;
    const double* B; int64_t sbk, sbn;
    double* C; int64_t ldc;
    int batch; int64_t strideA, strideB, strideC;
    // two-level batch: b -> (b / batch_inner, b % batch_inner); the *2 strides apply to the inner index
    int batch_inner = 1; int64_t strideA2 = 0, strideB2 = 0, strideC2 = 0;
    // optional restriction of the contraction range per output tile (operands with triangular zeros):
    // k_lo = max(klo_m ? tile row start : 0, klo_n ? tile col start : 0)
    // k_hi = min(khi_m ? tile row end : K, khi_n ? tile col end : K); tiles with k_lo >= k_hi write beta*C.
    int klo_m = 0, klo_n = 0, khi_m = 0, khi_n = 0;
    int skip_lower = 0;  // skip tiles entirely below the diagonal (col end <= row start): left untouched
    int skip_upper = 0;  // skip tiles entirely above the diagonal (row end <= col start)
    int skip_col0 = 0;   // column of C's first column relative to its first row, for the two tests above
    int diag_order = 0;  // rotate the tile columns of tile row r by r: spreads column-dependent contraction lengths over the XCDs
    const int* m_limit = nullptr;   // device array [batch]: rows m >= m_limit[b] of batch entry b are not computed
    // optional second pair of operands with the shapes, strides and batch strides of the first:
    // C = alpha (A B + A2 B2) + beta C in one pass (not combined with the contraction-range restrictions)
    const double* A2 = nullptr; const double* B2 = nullptr;
    int tag = -1;   // tboa_prof_tag of this launch (timed with HIP events when profiling is on)
};
int gemm_f64(tboa_ctx* ctx, const GemmF64& g);
// brackets a tagged launch with HIP events on the context's current stream when profiling is on
int prof_begin(tboa_ctx* ctx, int tag, double flops, ProfRec& rec, bool& timed);
int prof_end(tboa_ctx* ctx, const ProfRec& rec, bool timed);

// ---------------------------------------------------------------- gemm_bf16.hip
struct GemmBf16 {
    int M, N, K;
    float alpha;
    const __hip_bfloat16* A; int64_t lda;
    const __hip_bfloat16* B; int64_t ldb;
    void* C; int64_t ldc; int c_dtype; int accumulate; int flags;
    void* C2 = nullptr;   // with TBOA_GEMM_C_HILO: second 16-bit result buffer (the low parts), laid out as C
    float lo_scale = 1.f; // with TBOA_GEMM_C_HILO_HALF: the low parts are stored times this (a power of two that keeps them normal numbers)
    int batch; int64_t strideA, strideB, strideC;
    // two-level batch: z -> (z / batch_inner, z % batch_inner); the *2 strides apply to the inner index
    int batch_inner = 1; int64_t strideA2 = 0, strideB2 = 0, strideC2 = 0;
    int tag = -1;   // tboa_prof_tag of this launch (timed with HIP events when profiling is on)
    int kseg = 0;   // > 0: K is a concatenation of K/kseg segments; TBOA_GEMM_CAUSAL_K then limits each segment
    // nterms > 1 (persistent kernel only): the contraction runs over nterms operand pairs, K / nterms columns each, the
    // t-th pair read from termA[t], termB[t] (laid out and strided as A and B; A = termA[0], B = termB[0]):
    // C = sum_t termA[t] termB[t]^T in one pass over the accumulators
    int nterms = 1; const __hip_bfloat16* termA[4] = {}; const __hip_bfloat16* termB[4] = {};
};
// internal flag: a 16-bit result leaves as an exact-to-16-bit pair of bf16 values (hi into C, lo into C2), whatever the operands
#define TBOA_GEMM_C_HILO 0x10000
#define TBOA_GEMM_C_HILO_HALF 0x20000     // (with C_HILO) the pair is IEEE half, 22 significant bits, instead of bf16, 16: for values known to fit half
int gemm_bf16_nt(tboa_ctx* ctx, const GemmBf16& g);

// Transposed causal attention probabilities of all heads of one sequence as (hi, lo) pairs of 16-bit values (IEEE half
// when f16, else bf16): Pt[g][i][r L + t] = A_h[t, i], h = g rep + r, every [L, ldp] matrix of a KV group in 16 x 32 blocks,
// rows i up to the end of the 256-tile that holds t written (zeros beyond the diagonal).  dhi, dlo: A - A~ of a second
// score matrix (nullptr without one).
struct PtOut { __hip_bfloat16 *hi, *lo, *dhi, *dlo; };
// factor on the probabilities attn_probs_t / attn_probs_rows write as IEEE half (f16 set); bf16 results are unscaled
#define ATTN_PROBS_HALF_SCALE 16384.f
// How the (hi, lo) pairs of Q^ and K^ are encoded, per score matrix: a device word per operand that holds the bits of the
// largest magnitude of that operand's fp32 values, in which case the pairs are IEEE half values of the operand times
// 2^tboa_half_exp(word) (22 significant bits wherever the magnitude is within 2^-17 of the largest), or a negative word / a
// null pointer: pairs of bf16, unscaled (16 significant bits).
struct QkScale { const int *qa, *ka, *qb, *kb; };
// e such that amax 2^e lies in [2^13, 2^14) (amax: the bits of a non-negative float); 0 for zero, denormal or non-finite amax
__host__ __device__ __forceinline__ int tboa_half_exp(int amax_bits) {
    const int E = (amax_bits >> 23) & 0xff;
    return (E < 13 || E == 255) ? 0 : 140 - E;
}
// straight from the blocked 3-term operands Q^ [Hq][L, 3 dh], K^ [Hkv][L, 3 dh] of the score product (second pair Qb, Kb or
// nullptr); attn_probs_t_supported tells which shapes the kernel takes
bool attn_probs_t_supported(int L, int dh);
// the same probabilities with the queries as rows, P[h][t][.] = [A_hi | A_lo | A~_hi | A~_lo] (segments of L columns, pitch ldp, a
// multiple of 32: every head's [L, ldp] matrix in 16 x 32 blocks; the last two segments only with a second pair: the
// probabilities of the second score matrix), rows written up to the end of the 256-tile of t
int attn_probs_rows(tboa_ctx* ctx, const __hip_bfloat16* Qa, const __hip_bfloat16* Ka, const __hip_bfloat16* Qb, const __hip_bfloat16* Kb, int L,
                    int Hq, int rep, int dh, __hip_bfloat16* P, long long ldp, int f16, QkScale qs);
int attn_probs_t(tboa_ctx* ctx, const __hip_bfloat16* Qa, const __hip_bfloat16* Ka, const __hip_bfloat16* Qb, const __hip_bfloat16* Kb, int L,
                 int Hq, int rep, int dh, PtOut out, long long ldp, long long group_stride, int f16, QkScale qs);

// element offset of (r, c) in a matrix kept in the 16 x 32 blocks the bf16 GEMM can read and write (TBOA_GEMM_*_TILED);
// kb = leading dimension / 32
__device__ __forceinline__ long long tboa_blocked_offset(long long r, long long c, long long kb) {
    const int ri = (int)(r & 15), ci = (int)(c & 31);
    return ((r >> 4) * kb + (c >> 5)) * 512 + ri * 32 + (((ci >> 3) ^ (ri >> 2)) << 3) + (ci & 7);
}

// ---------------------------------------------------------------- factor.hip
// H64 [batch, n, n] fp64, overwritten; U [batch, n, n] fp64 out.  Checks the device status and
// returns TBOA_ENOTSPD on breakdown (synchronises).  tmp: workspace of batch * n * chol_tmp_pitch(n) doubles,
// dinv: batch * ceil(n / TB_FACT_NB) * TB_FACT_NB^2 doubles.
#define TB_FACT_NB 64     // diagonal blocks factored inside LDS
#define TB_FACT_OB 512    // outer blocks: width of the large trailing updates
static inline int chol_tmp_pitch(int n) { return n <= TB_FACT_OB ? TB_FACT_NB : TB_FACT_OB; }
// status_slot: which pair of device status words records a breakdown (0 or 2); defer_status: do not wait for them here,
// the caller checks with chol_status_f64 once the work has been joined.
int chol_inv_upper_f64(tboa_ctx* ctx, int n, int batch, double* H64, double* U, double* tmp, double* dinv, int status_slot = 0,
                       bool defer_status = false);
int chol_status_f64(tboa_ctx* ctx, int status_slot);
int chol_static_init(int device);   // looks up the device address of the static scratch of tboa_chol_inv_upper_static (device current)
int launch_f32_to_f64_damp(tboa_ctx* ctx, int n, int batch, const float* H, double damp, double* out);

// ---------------------------------------------------------------- misc elementwise (elementwise.hip)
int launch_fill_f64(tboa_ctx* ctx, double* p, int64_t n, double v);
int launch_fill_f32(tboa_ctx* ctx, float* p, int64_t n, float v);
int launch_cvt_to_f64(tboa_ctx* ctx, const void* src, int dtype, double* dst, int64_t n);
int launch_cvt_f64_to_f32(tboa_ctx* ctx, const double* src, float* dst, int64_t n);
int launch_cvt_f32_to_f64(tboa_ctx* ctx, const float* src, double* dst, int64_t n);
// out[r, c] = in[r, c] for c > r else 0 (square n x n, batch)
int launch_strict_upper_f64(tboa_ctx* ctx, double* a, int n, int batch);
// symmetrise: upper <- lower (fp32, n x n, batch)
int launch_mirror_lower_f32(tboa_ctx* ctx, float* a, int n, int batch);
int launch_sub_f64(tboa_ctx* ctx, const double* a, const double* b, double* out, int64_t n);

// ---------------------------------------------------------------- hessian_f64.hip
int build_hessians_f64(tboa_ctx* ctx, const tboa_attn_desc* d, const void* X, const void* X_fp, const void* Wq, const void* Wk,
                       const void* Wv, const void* Wo, float* Hin_qk, float* R_qk, float* Hout_q, float* Hout_k, float* Hin_v,
                       float* R_v, float* Hout_v);
int build_hessian_out_proj_f64(tboa_ctx* ctx, const tboa_attn_desc* d, const void* X, const void* X_fp, const float* Wq_deq,
                               const float* Wk_deq, const float* Wv_deq, const void* Wq, const void* Wk, const void* Wv,
                               float* Hin_o, float* R_o);
int build_hessian_linear_f64(tboa_ctx* ctx, long long T, int n, double alpha, const float* X, const float* X_fp, float* H_in, float* R);
int attention_forward_f64(tboa_ctx* ctx, const tboa_attn_desc* d, const float* X, const float* Wq, const float* Wk, const float* Wv, float* O);
int linear_forward_f64(tboa_ctx* ctx, long long T, int din, int dout, const float* X, const float* W, const float* Res, float* Y);
int swiglu_forward_f64(tboa_ctx* ctx, long long T, int d, int dff, const float* X, const float* Wg, const float* Wu, float* Act);
