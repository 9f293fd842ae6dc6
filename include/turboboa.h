/*
 * turboboa.h — C ABI of the TurboBoA quantization hot path for one attention block on MI355X.
 *
 * The library quantizes the projection weights of one attention block (W_Q, W_K, W_V, W_O) with the
 * TurboBoA procedure (Algorithm 1 of the paper): Kronecker-factored attention-aware Hessians
 * H = H_in (x) H_out (Table 1), U = Chol(H^-1)^T (eq. 3), joint quantization of N out-channels per
 * sequential step with the closed-form compensation of the remaining out-channels (Prop. 3.1), the
 * correction for errors propagated from earlier quantized layers (Prop. 3.2, R = alpha dX X^T), a grid
 * recomputed for the rows of each step (Sec. 3.3), the in-channel sweep of Algorithm 3 and the
 * coordinate-descent scale refinement of Prop. 3.3 / Algorithm 2.
 *
 * Conventions
 *   - Every tensor pointer is DEVICE memory owned by the caller unless marked "host".  Inputs are never
 *     modified; the library keeps no pointer after a call returns.  Temporary storage belongs to the
 *     context: one workspace, grown on demand (a growth frees and reallocates it after synchronising the stream) and
 *     released by tboa_destroy.  tboa_hessian_workspace_bytes / tboa_quantize_workspace_bytes tell what a call will need
 *     and tboa_reserve_workspace obtains it ahead, so that no call allocates afterwards.
 *   - Matrices are dense row-major.  Activations are token-major: X[t, c] is channel c of token t, so the
 *     paper's X (channels x tokens) is the transpose and H_in = X X^T = sum_t x_t x_t^T.
 *     Weights are [out-channels, in-channels]; head h of a projection owns rows h*d_h .. (h+1)*d_h-1.
 *   - All work is enqueued on the stream given to tboa_create; a call that returns values or a status read from the
 *     device (tboa_quantize_layer: factorisation breakdown, losses) synchronises that stream once, at its end.
 *   - Every function returns 0 on success or a negative tboa_status; tboa_last_error() then describes it.
 *     No exceptions, no abort, nothing printed.  One context per host thread.
 */
#ifndef TURBOBOA_H
#define TURBOBOA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tboa_ctx tboa_ctx;

enum tboa_status {
    TBOA_OK = 0,
    TBOA_EINVAL = -1,   /* null pointer, bad shape, unsupported parameter              */
    TBOA_ENOTSPD = -2,  /* a Hessian is not positive definite (non-positive pivot)     */
    TBOA_ENOMEM = -3,   /* workspace allocation failed                                  */
    TBOA_EHIP = -4,     /* a HIP call failed (message carries hipGetErrorString)        */
    TBOA_ENAN = -5      /* non-finite value met where a finite one is required          */
};

enum tboa_dtype { TBOA_F32 = 0, TBOA_BF16 = 1, TBOA_F64 = 2 };

/* Creates a context bound to HIP device `hip_device`; all kernels run on `hip_stream`
 * (a hipStream_t, e.g. torch.cuda.current_stream().cuda_stream; NULL = the default stream).
 * The context also owns one more stream of default priority on which tboa_quantize_layer runs work that is independent of
 * what `hip_stream` is doing; it is forked from and joined back into `hip_stream` inside the call, so that for the caller
 * everything still happens on `hip_stream` in call order. */
int tboa_create(tboa_ctx** out, int hip_device, void* hip_stream);
void tboa_destroy(tboa_ctx* ctx);
/* Text of the last error on this context; owned by the context, valid until the next call on it. */
const char* tboa_last_error(const tboa_ctx* ctx);
/* Event counters of this context since its creation (host values).
 * TBOA_CTR_GRID_PASSES: grid-search passes that used the two-phase search (approximate costs of all candidates on the
 * bf16 matrix cores, exact fp64 costs of the near-minimal ones); TBOA_CTR_GRID_FALLBACKS: tboa_quantize_layer calls whose
 * two-phase search did not trust itself (see tboa_layer_desc.grid_guard) and that were therefore run again with every
 * candidate of every row evaluated in fp64; TBOA_CTR_GRID_EXACT_ROWS: unused, always 0;
 * TBOA_CTR_GRID_SURVIVORS: near-minimal candidates that were evaluated exactly (rows with a single near-minimal
 * candidate need none).
 * TBOA_CTR_WEIGHTS_INT_FORM / TBOA_CTR_WEIGHTS_HILO: dequantized fp32 weight matrices handed to
 * tboa_build_hessian_out_proj or tboa_swiglu_forward that were found to be integer multiples of one step per row (one
 * bf16 GEMM with exact operands per product) / that were not and were split into bf16 terms (two or three). */
enum tboa_counter_id { TBOA_CTR_GRID_PASSES = 0, TBOA_CTR_GRID_FALLBACKS = 1, TBOA_CTR_GRID_EXACT_ROWS = 2, TBOA_CTR_GRID_SURVIVORS = 3,
                       TBOA_CTR_WEIGHTS_INT_FORM = 4, TBOA_CTR_WEIGHTS_HILO = 5 };
int64_t tboa_counter(const tboa_ctx* ctx, int which);
/* Bytes of context-owned workspace currently allocated (host value). */
size_t tboa_workspace_bytes(const tboa_ctx* ctx);
/* Makes the context's workspace at least `bytes` large (no-op when it already is).  Synchronises the stream when it has to
 * reallocate.  TBOA_ENOMEM when the device cannot provide it (the context then has no workspace at all). */
int tboa_reserve_workspace(tboa_ctx* ctx, size_t bytes);

/* ------------------------------------------------------------------------------------------------
 * Attention block description (Algorithm 1 inputs).  T = n_seqs * seq_len tokens.
 * GQA: query head h uses KV head h / (n_q_heads / n_kv_heads).
 */
typedef struct {
    int d_model, n_q_heads, n_kv_heads, head_dim, n_seqs, seq_len;
    int x_dtype;   /* tboa_dtype of X, X_fp and of the weights: TBOA_F32 or TBOA_BF16.
                      TBOA_BF16: contractions run on bf16 MFMA with fp32 accumulation (operands are exact).
                      TBOA_F32: contractions run on fp64 MFMA (small problems, reference-grade accuracy). */
    int causal;    /* 1: causal mask inside A_h = softmax(Q_h K_h^T / sqrt(d_h)) */
    double alpha;  /* stabilisation coefficient of Algorithm 1 line 5; R = alpha (X - X_fp) X^T */
    int seq_chunk; /* sequences processed per pass of the W_V Hessian (0 = library default) */
} tboa_attn_desc;

/* Table 1 Hessian factors of W_Q,h / W_K,g / W_V,g and the deviation correlations R (Algorithm 1,
 * lines 4-5).  Literal sums over all tokens, no normalisation, no damping.
 *   X      [T, d_model]  input of the (partly quantized) model            (x_dtype)
 *   X_fp   [T, d_model]  input of the full-precision model, or NULL: then R_qk and R_v are not written
 *   Wq [Hq*dh, d], Wk, Wv [Hkv*dh, d], Wo [d, Hq*dh]                     (x_dtype)
 * Outputs (fp32, caller-allocated):
 *   Hin_qk [d, d]        = sum_t x_t x_t^T                    (H_in of W_Q and W_K)
 *   R_qk   [d, d]        = alpha * sum_t (x_t - x~_t) x_t^T   (rows index the deviation)
 *   Hout_q [Hq, dh, dh]  = K_g(h)^T K_g(h)
 *   Hout_k [Hkv, dh, dh] = sum over query heads of the group of Q_h^T Q_h
 *   Hin_v  [Hkv, d, d]   = sum over query heads of the group and sequences of (A_h X_s)^T (A_h X_s)
 *   R_v    [Hkv, d, d]   = alpha * sum (A_h X_s - A~_h X~_s)^T (A_h X_s), or NULL to skip
 *   Hout_v [Hkv, dh, dh] = sum over query heads of the group of W_out,h^T W_out,h
 * The outputs come in independent parts, and a part whose pointers are NULL is not computed: {Hin_qk, Hout_q, Hout_k
 * (+ R_qk)} (all three or none), {Hin_v (+ R_v)} (by far the most expensive part), {Hout_v}.  A caller may so obtain the
 * factors of W_Q and W_K first and quantize them on other streams while the W_V part is still being built.
 *   fp_cache  NULL, or caller-allocated device memory of tboa_fp_cache_bytes(desc) bytes (16-byte aligned; needs R_v):
 *             receives the projections of X_fp by the full-precision W_Q and W_K (an opaque layout), which both this call
 *             and tboa_build_hessian_out_proj need for their deviation terms; handing the buffer to the latter saves it two
 *             projections per token.  Valid for the (desc, X_fp, Wq, Wk) of this call.  Used on the bf16 path only
 *             (tboa_fp_cache_bytes is 0 for fp32 inputs: pass NULL).
 */
size_t tboa_fp_cache_bytes(const tboa_attn_desc* desc);
/* Workspace that tboa_build_hessians and tboa_build_hessian_out_proj need for this block (the larger of the two, with X_fp
 * and every output requested); 0 for an invalid descriptor. */
size_t tboa_hessian_workspace_bytes(const tboa_attn_desc* desc);
int tboa_build_hessians(tboa_ctx* ctx, const tboa_attn_desc* desc,
                        const void* X, const void* X_fp,
                        const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                        float* Hin_qk, float* R_qk, float* Hout_q, float* Hout_k,
                        float* Hin_v, float* R_v, float* Hout_v, void* fp_cache);

/* Hessian of the output projection: the layer-wise row of Table 1, X_o X_o^T (x) I, with X_o the
 * attention output concat_h(A_h V_h) computed from the DEQUANTIZED W_Q, W_K, W_V (fp32 [.., d]) on X;
 * R_o = alpha (X_o - X~_o) X_o^T with X~_o from the full-precision weights (x_dtype) on X_fp.
 *   Hin_o [Hq*dh, Hq*dh] fp32;  R_o same shape or NULL (then X_fp, Wq, Wk, Wv may be NULL).
 * On the bf16 path a dequantized weight whose rows are integer multiples (|k| <= 256) of one step per row, as the W_deq
 * of tboa_quantize_layer with per-row grids is, enters its products as those integers (exact in bf16) with the steps
 * applied to the result; any other fp32 weight as three bf16 terms that carry its 24 bits.  Synchronises the stream.
 *   fp_cache  NULL, or the buffer a tboa_build_hessians call with the same desc, X_fp, Wq, Wk filled (bf16 path, R_o
 *             requested): the projections of X_fp are then read from it and Wq, Wk may be NULL.
 */
int tboa_build_hessian_out_proj(tboa_ctx* ctx, const tboa_attn_desc* desc,
                                const void* X, const void* X_fp,
                                const float* Wq_deq, const float* Wk_deq, const float* Wv_deq,
                                const void* Wq, const void* Wk, const void* Wv,
                                float* Hin_o, float* R_o, const void* fp_cache);

/* Gated MLP of the same transformer block (W_gate, W_up: [d_ff, d]; W_down: [d, d_ff]).  Its three projections are plain
 * linear layers: the layer-wise row of Table 1 (H = X X^T (x) I, no out-channel coupling), quantized by
 * tboa_quantize_layer with H_out = NULL, and with the deviation correlation R of Prop. 3.2 when the input of the
 * full-precision model is given.
 *   X, X_fp [n_tokens, d_in] (x_dtype; X_fp and R both NULL or both given)
 *   H_in [d_in, d_in] = sum_t x_t x_t^T,  R [d_in, d_in] = alpha sum_t (x_t - x~_t) x_t^T   (fp32, caller-allocated) */
int tboa_build_hessian_linear(tboa_ctx* ctx, int64_t n_tokens, int d_in, int x_dtype, double alpha,
                              const void* X, const void* X_fp, float* H_in, float* R);
/* Input of the down projection: Act = silu(X W_gate^T) * (X W_up^T), silu(g) = g / (1 + exp(-g)).
 *   X [n_tokens, d] (x_dtype); W_gate, W_up [d_ff, d] in w_dtype: x_dtype, or TBOA_F32 for dequantized weights (on the
 *   bf16 path used in integer form or as (hi, lo) bf16 pairs, as in tboa_build_hessian_out_proj);
 *   Act [n_tokens, d_ff] (x_dtype). */
int tboa_swiglu_forward(tboa_ctx* ctx, int64_t n_tokens, int d, int d_ff, int x_dtype, const void* X,
                        int w_dtype, const void* W_gate, const void* W_up, void* Act);

/* Out-channel Hessian factor of a projection whose partner is given as a weight matrix (Table 1 without positional rotation:
 * K_g^T K_g = W_K,g H_in W_K,g^T and likewise for Q):  H_out[g] = sum over the `rep` consecutive heads h of group g of W_h H_in W_h^T,
 * W_h = rows h*head_dim .. of W.  With W = the DEQUANTIZED W_Q (w_dtype TBOA_F32) and rep = Hq / Hkv this is the H_out of W_K as
 * Algorithm 1 computes it when its Hessians are formed inside the loop over the layers (line 4), after W_Q has been quantized;
 * with W = W_K and rep = 1 it is the H_out of W_Q (per KV head).  H_in [d_in, d_in] fp32 (undamped), W [n_heads*rep*head_dim, d_in]
 * in w_dtype (TBOA_F32 or TBOA_BF16), H_out [n_heads, head_dim, head_dim] fp32.  fp64 arithmetic. */
int tboa_build_hout(tboa_ctx* ctx, int d_in, int n_heads, int rep, int head_dim, const float* H_in, int w_dtype, const void* W,
                    float* H_out);

/* H_out of W_Q,h when the keys are held in a kv_bits-bit cache (Sec. 4.2, the setting with a quantized KV cache): G = K^_g in
 * the W_Q row of Table 1, K^_g the per-token Min-Max fake-quant of the head vectors k_{g,t} = W_K,g x_t (the quantizer of
 * tboa_act_fakequant with one scale and zero per token and KV head; levels decided in fp64).  X [n_seqs*seq_len, d_model] and
 * W_K [n_kv_heads*head_dim, d_model] in desc->x_dtype; Hout_q [n_q_heads, head_dim, head_dim] fp32, the literal sum of
 * k^ k^^T over all tokens, every query head of a KV group receiving its group's matrix.  kv_bits in 2 .. 8.  Nothing else of
 * the Hessians changes with it: a caller replaces the Hout_q of tboa_build_hessians by this one. */
int tboa_build_hout_q_kv_cache(tboa_ctx* ctx, const tboa_attn_desc* desc, const void* X, const void* Wk, int kv_bits, float* Hout_q);

/* Forward pass of the block, for the driver that carries the two activation streams from one transformer block to the next
 * (Sec. 3.2: the deviation that Prop. 3.2 corrects is the one accumulated through the preceding quantized layers):
 * tboa_attention_forward: O[t, h dh + c] = sum_k A_h[t, k] V_g(h)[k, c], A_h = softmax(Q_h K_g^T / sqrt(d_h)) per sequence (the input of
 *   the output projection).  X [T, d_model] (x_dtype); Wq [Hq dh, d], Wk, Wv [Hkv dh, d] in w_dtype: x_dtype, or TBOA_F32 for
 *   dequantized weights; O [T, Hq dh] (x_dtype).  bf16 path: same products as tboa_build_hessian_out_proj (synchronises).
 * tboa_linear_forward: Y = X W^T (+ Res).  X [n_tokens, d_in], Res (or NULL) and Y [n_tokens, d_out] in x_dtype; W [d_out, d_in] in
 *   w_dtype (x_dtype or TBOA_F32). */
int tboa_attention_forward(tboa_ctx* ctx, const tboa_attn_desc* desc, const void* X, int w_dtype, const void* Wq, const void* Wk,
                           const void* Wv, void* O);
int tboa_linear_forward(tboa_ctx* ctx, int64_t n_tokens, int d_in, int d_out, int x_dtype, const void* X, int w_dtype, const void* W,
                        const void* Res, void* Y);

/* Min-Max dynamic per-token activation quantizer (weight-activation experiments): one asymmetric
 * (scale, zero) per token from that token's min and max, `bits` levels; writes the dequantized
 * activations.  X_in, X_out [T, d] in `dtype` (TBOA_F32 or TBOA_BF16); may alias. */
int tboa_act_fakequant(tboa_ctx* ctx, int64_t n_tokens, int d, int bits, int dtype,
                       const void* X_in, void* X_out);

/* Randomised Hadamard rotation of activations, the fixed training-free transform that the weight-activation
 * experiments apply before quantization to spread outlier channels (Sec. 4.2 with App. B):
 *   X_out[t, :] = (X_in[t, :] * signs) H_d / sqrt(d),  H_d[i, j] = (-1)^popcount(i & j)  (Sylvester-Hadamard, d = 2^k).
 * X_in, X_out [n_tokens, d] in `dtype` (TBOA_F32 or TBOA_BF16; may alias; 16-byte aligned, signs too), arithmetic in fp32;
 * signs: d floats, each +1 or -1, or NULL (all +1).  d must be a power of two in 16 .. 16384. */
int tboa_hadamard_rotate(tboa_ctx* ctx, int64_t n_tokens, int d, int dtype, const void* X_in, const float* signs, void* X_out);

/* ------------------------------------------------------------------------------------------------
 * One projection weight (Algorithm 1 lines 2-13).
 */
typedef struct {
    int d_out, d_in;
    int n_heads;        /* d_out = n_heads * d_h; heads are independent                               */
    int hin_per_head;   /* 0: H_in, R are [d_in, d_in]; 1: [n_heads, d_in, d_in] (W_V)                */
    int bits;           /* 2, 3, 4 or 8                                                               */
    int block;          /* N: out-channels quantized jointly per sequential step (ragged last block)  */
    int group;          /* 0: one (scale, zero) per row; g > 0: per g consecutive in-channels, g | d_in */
    int w_dtype;        /* tboa_dtype of W: TBOA_F32 or TBOA_BF16                                      */
    int cd_iters;       /* n_iter of Algorithm 2 (paper: 1); 0 disables the refinement                */
    int adaptive_grid;  /* 1: grid recomputed for the rows of each step (Algorithm 1 line 9);
                           0: one grid from the original weights, kept fixed (BoA)                    */
    int grid_points;    /* candidates per unit shrink (100)                                           */
    double max_shrink;  /* candidates k = 0 .. ceil(max_shrink*grid_points)-1, range scaled by 1-k/grid_points */
    double damp;        /* every Hessian gets damp * mean(diag) added to its diagonal at entry        */
    double grid_guard;  /* the grid search of wide per-row layers (d_in >= 256, group = 0) finds its candidates' costs
                           approximately on the bf16 matrix cores and re-evaluates the near-minimal ones (within tau = 2e-3
                           of the minimum) in fp64; every re-evaluation is compared with its approximation, and a call in
                           which one differs by more than grid_guard * tau (relative) is run again with fp64 costs for every
                           candidate.  0: the default, 0.25.  Negative: fp64 costs for every candidate from the start. */
} tboa_layer_desc;

/* Workspace that tboa_quantize_layer needs for this descriptor, called with (with_H_out != 0) or without H_out and with
 * (with_R != 0) or without R; 0 for an invalid descriptor.  (Without H_out the rows are independent, and the group-wise
 * scale refinement then keeps one Gram entry per row and pair of groups instead of one d_h x d_h block per head.) */
size_t tboa_quantize_workspace_bytes(const tboa_layer_desc* desc, int with_H_out, int with_R);

/*   W      [d_out, d_in]            (w_dtype)
 *   H_in   fp32, shape per hin_per_head
 *   H_out  [n_heads, d_h, d_h] fp32, or NULL = identity (output projection / GPTQ: rows decouple,
 *          no compensation between out-channels)
 *   R      fp32, same shape as H_in, already scaled by alpha, or NULL = 0 (first block / BoA)
 * Outputs:
 *   codes  [d_out, d_in] uint8, one code per byte, 0 .. 2^bits-1
 *   scales, zeros [d_out, n_groups] fp32 (n_groups = 1 or d_in/group); zeros hold integer values
 *   W_deq  [d_out, d_in] fp32 = scales * (codes - zeros)
 *   loss   host double[2] or NULL: {tr(H_out D H_in D^T), 2 tr(H_out W R D^T)} summed over heads, D = W_deq - W,
 *          on the damped Hessians (the D-dependent part of the attention reconstruction error)
 *   loss_per_head  host double[n_heads][2] or NULL: the two terms of every head
 * Synchronises the stream once, at the end (breakdown status of the factorisations, the losses, the guard of the grid search).
 */
int tboa_quantize_layer(tboa_ctx* ctx, const tboa_layer_desc* desc,
                        const void* W, const float* H_in, const float* H_out, const float* R,
                        uint8_t* codes, float* scales, float* zeros, float* W_deq,
                        double* loss, double* loss_per_head);

/* ------------------------------------------------------------------------------------------------
 * Deployable form of the result (the reduced memory footprint is the purpose of weight quantization, Sec. 1).
 * The codes of a row form a little-endian bit stream: code c occupies bits [bits*c, bits*c + bits) of the stream, which is
 * stored as 32-bit words (bit i of the stream = bit i % 32 of word i / 32); every row starts on a word and is padded
 * with zero bits to tboa_packed_words_per_row(d_in, bits) = ceil(d_in * bits / 32) words.  A 3-bit code may straddle two
 * words.  bits in {2, 3, 4, 8}.
 */
int64_t tboa_packed_words_per_row(int d_in, int bits);   /* host value, no context needed; 0 for non-positive arguments */
/*   codes  [d_out, d_in] uint8 (as written by tboa_quantize_layer)  ->  packed [d_out, words_per_row] uint32 */
int tboa_pack_codes(tboa_ctx* ctx, int d_out, int d_in, int bits, const uint8_t* codes, uint32_t* packed);
/* y = W_deq x from the packed form alone: y[r] = sum_c scales[r, c/g] (code[r, c] - zeros[r, c/g]) x[c].
 *   packed as above; scales, zeros [d_out, n_groups] fp32 (group = 0: one group per row); x [d_in], y [d_out] fp32.
 * A check that the packed codes, scales and zeros carry the quantized layer; accumulation in fp64. */
int tboa_dequant_gemv(tboa_ctx* ctx, int d_out, int d_in, int bits, int group, const uint32_t* packed,
                      const float* scales, const float* zeros, const float* x, float* y);

/* ------------------------------------------------------------------------------------------------
 * Building blocks, exported for stage-isolated checks and for roofline measurement.
 */

/* U = Chol(H^-1)^T (eq. 3): upper triangular, H^-1 = U^T U, for `batch` matrices of order n.
 * H fp32 [batch, n, n] (only read); damp as in tboa_layer_desc; U fp64 [batch, n, n] (strict lower part zero). */
int tboa_chol_inv_upper(tboa_ctx* ctx, int n, int batch, const float* H, double damp, double* U);

/* tboa_chol_inv_upper for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): same arguments, same kernels, same result, but the temporaries live in a static device
 * array of 24 MiB that every GPU the library runs on holds until the process ends (its address is looked up by
 * tboa_create), not in the context's workspace.  The call allocates and frees nothing.
 * Limits: n <= 512 and batch * roundup64(n)^2 <= tboa_chol_inv_upper_static_max_elems() (= 2^20; e.g. 64 matrices of order
 * 128, 4 of order 512); larger requests return TBOA_EINVAL with a message and touch nothing.
 * All calls on one GPU share the array, which keeps the last call's contents (nothing in it needs to start at zero: every
 * part is written before it is read): calls that overlap in time on the same GPU race, on whatever streams or contexts. */
size_t tboa_chol_inv_upper_static_max_elems(void);
int tboa_chol_inv_upper_static(tboa_ctx* ctx, int n, int batch, const float* H, double damp, double* U);

/* C[b] = alpha * A[b] B[b] + beta * C[b] in fp64 on the fp64 matrix cores.
 * A(m,k) = A[m*sam + k*sak], B(k,n) = B[k*sbk + n*sbn]; in each pair one stride must be 1. C row-major, ldc. */
int tboa_gemm_f64(tboa_ctx* ctx, int M, int N, int K, double alpha,
                  const double* A, int64_t sam, int64_t sak, const double* B, int64_t sbk, int64_t sbn,
                  double beta, double* C, int64_t ldc,
                  int batch, int64_t strideA, int64_t strideB, int64_t strideC);

/* C[b] = alpha * A[b] B[b]^T (+ C[b] if accumulate) with bf16 operands, fp32 accumulation on the bf16
 * matrix cores.  A [M, K] row-major lda, B [N, K] row-major ldb (both K-contiguous; lda, ldb multiples of 8,
 * pointers 16-byte aligned).  C [M, N] ldc, fp32 (c_dtype = TBOA_F32) or bf16 (TBOA_BF16, accumulate must be 0).
 * flags: TBOA_GEMM_LOWER computes only tiles on or below the diagonal (M == N; a symmetric product),
 *        TBOA_GEMM_CAUSAL_K limits the contraction of output column n to k <= n rounded up to the tile
 *        (B is lower triangular: causal attention probabilities),
 *        TBOA_GEMM_PERSISTENT runs one resident workgroup per compute unit over a precomputed list of tiles instead of
 *        one dispatched workgroup per tile (same arithmetic, same result; taken when the contraction length, or kseg, is
 *        a multiple of 128, ignored otherwise).  Meant for launches that have the GPU to themselves: the lists are
 *        balanced for compute units that all start together.
 *        TBOA_GEMM_A_TILED / _B_TILED / _C_TILED: that matrix is not row-major but stored in blocks of 16 rows x 32 columns
 *        (1 KB, the unit the kernel copies into LDS with one wavefront load): element (r, c) of a matrix with leading
 *        dimension ld (a multiple of 32) sits at element offset
 *            ((r / 16) * (ld / 32) + c / 32) * 512 + (r % 16) * 32 + (((c % 32) / 8) ^ (((r % 16) / 4) % 4)) * 8 + c % 8,
 *        i.e. the blocks of a block row follow each other along the columns and the four 16-byte pieces of a row of a
 *        block are XOR-permuted the way the kernel keeps them in LDS.  A column offset c0 (a multiple of 32) into such a
 *        matrix is the pointer offset 16 * c0.  Operands: rows a multiple of 16, K a multiple of 32 (batch strides as for
 *        row-major operands; blocks that start on 128-byte boundaries are read as whole cache lines); C: bf16, no
 *        accumulation, M and N multiples of 256.  Meant for chains of products where one
 *        product's bf16 result is the next one's operand (its loads are then whole contiguous blocks).
 *        TBOA_GEMM_KLO: the contraction of the output tile at (m0, n0) starts at k = max(m0, n0) (tile starts, multiples of
 *        256) in every segment: for operands with A[m, k] = 0 for k < m and B[n, k] = 0 for k < n, such as transposed causal
 *        attention probabilities (contraction or segment length a multiple of 256, M and N not larger).
 *        TBOA_GEMM_F16: A and B (and a C of c_dtype TBOA_BF16, i.e. 16 bits wide) hold IEEE half values instead of bf16:
 *        same layouts, same rate, 11 instead of 8 significant bits, range up to 65504. */
enum { TBOA_GEMM_LOWER = 1, TBOA_GEMM_CAUSAL_K = 2, TBOA_GEMM_PERSISTENT = 4, TBOA_GEMM_A_TILED = 8, TBOA_GEMM_B_TILED = 16,
       TBOA_GEMM_C_TILED = 32, TBOA_GEMM_F16 = 64, TBOA_GEMM_KLO = 128 };
int tboa_gemm_bf16_nt(tboa_ctx* ctx, int M, int N, int K, float alpha,
                      const void* A, int64_t lda, const void* B, int64_t ldb,
                      void* C, int64_t ldc, int c_dtype, int accumulate, int flags,
                      int batch, int64_t strideA, int64_t strideB, int64_t strideC);

/* ------------------------------------------------------------------------------------------------
 * Live kernel timing.  With profiling on, every GEMM launch that carries one of the tags
 * below is bracketed by HIP events on the stream it is launched on.  tboa_profile_read synchronises the stream and returns,
 * for one tag, the summed kernel time, the number of launches and the summed algorithmic flops of those launches
 * (2 M N K per batch entry; a symmetric product counts its M(M+1)/2 unique outputs, a product with a lower
 * triangular factor the k <= n part).  tboa_profile_reset drops the records.
 */
enum tboa_prof_tag {
    TBOA_PROF_HV_SYRK = 0,   /* H_in^V += Y^T (Y^T)^T                 */
    TBOA_PROF_AX = 1,        /* Y^T = X_s^T A_h^T (and the dY^T form) */
    TBOA_PROF_RV = 2,        /* R_v += alpha dY^T (Y^T)^T             */
    TBOA_PROF_GRAM = 3,      /* X X^T, dX X^T, O O^T over all tokens  */
    TBOA_PROF_PROJ = 4,      /* projections and scores                */
    TBOA_PROF_GRID = 5,      /* approximate grid-search costs (quantize_layer) */
    /* fp64 matrix-core GEMMs of tboa_quantize_layer (flops: 2 M N K over the contraction range every tile really has) */
    TBOA_PROF_F64_GRID = 6,    /* exact grid-search costs (near-minimal candidates: timed, flops not counted; or all candidates) */
    TBOA_PROF_F64_FACTOR = 7,  /* P = ((R U^T) * M_U) U of Algorithm 3                                    */
    TBOA_PROF_F64_SWEEP = 8,   /* rank-64 updates of the columns right of a panel of the in-channel sweep */
    TBOA_PROF_F64_COMP = 9,    /* compensation of the remaining out-channels (Prop. 3.1 / 3.2)            */
    TBOA_PROF_F64_CD = 10,     /* products of the scale refinement (Algorithm 2) and of the loss          */
    TBOA_PROF_ATA = 11,        /* sum over a KV group's heads of A_h^T A_h and A_h^T (A_h - A~_h) (grouped-query form of the W_V Hessian) */
    TBOA_PROF_SCORES = 12,     /* scores Q_h K_g^T of a sequence (short contraction: 3 d_h with the (hi, lo) parts), fp32 out */
    TBOA_PROF_PV = 13,         /* attention outputs O_h^T = V^T A_h^T and their differences, for the W_O Hessian */
    TBOA_PROF_NTAGS = 14
};
int tboa_profile_enable(tboa_ctx* ctx, int on);
int tboa_profile_reset(tboa_ctx* ctx);
int tboa_profile_read(tboa_ctx* ctx, int tag, double* ms_total, int64_t* launches, double* flops_total);

#ifdef __cplusplus
}
#endif
#endif /* TURBOBOA_H */
