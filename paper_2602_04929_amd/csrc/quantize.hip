// tboa_quantize_layer: Algorithm 1 (lines 2-13) for one projection weight, all arithmetic in fp64.
//
// Heads are independent and run side by side: the N rows of the current step of every head form one
// "block" of n_heads*N rows (block row R = h*nbr + r  <->  layer row h*d_h + i0 + r).  Per step:
//   grid search   (Alg. 1 line 9)  candidates -> approximate costs of all of them on the bf16 matrix cores (delta and H_in as
//                                  (hi, lo) bf16 pairs) -> exact fp64 costs of the near-minimal ones -> argmin
//                                  (narrow layers and group-wise grids: every candidate exactly, one fp64 GEMM)
//   in-channel sweep (Algorithm 3) panels of 64 columns: a wavefront owns a row, lane k holds column k, the 64
//                                  sequential column steps run inside the kernel with U/P panel rows in LDS;
//                                  columns right of the panel get one rank-64 GEMM update per term
//   compensation  (Prop. 3.1/3.2)  T = [U_out^T]_{i1:,B} [U_out^T]_{B,B}^-1 per head, then W~[i1:] -= T E as a
//                                  batched GEMM, E = (W_B - Q_B) - ((W_B R) U_in^T) U_in
// and after the last step the coordinate descent of Algorithm 2 on precomputed Gram matrices (d_h x d_h per head; per
// pair of groups when the grids are group-wise), then the outputs and the loss.
#include "internal.h"
#include <string.h>
#include <stdlib.h>
#include <math.h>

namespace {

struct BlockMap { int nbr, dh, i0; };
__device__ __forceinline__ long long layer_row(const BlockMap& m, int R) {
    return (long long)(R / m.nbr) * m.dh + m.i0 + (R % m.nbr);
}

__device__ __forceinline__ double readlane_f64(double v, int l) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_readlane(lo, l);
    hi = __builtin_amdgcn_readlane(hi, l);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ double quant_code(double w, double s, double z, double maxq) {
    return fmin(fmax(rint(w / s) + z, 0.0), maxq);
}

// ------------------------------------------------------------------------------------------------ rows
__global__ void gather_rows_kernel(const double* __restrict__ src, double* __restrict__ dst, BlockMap m, int n) {
    const int R = blockIdx.y;
    const double* s = src + layer_row(m, R) * n;
    double* d = dst + (long long)R * n;
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n; c += gridDim.x * blockDim.x) d[c] = s[c];
}

// ------------------------------------------------------------------------------------------------ grid search
// one wavefront per row: range of the row, then the candidate list (s_k, z_k)
__global__ __launch_bounds__(256) void grid_candidates_kernel(const double* __restrict__ Wk, long long ldw, int c0, int ncols,
                                                              int rows, int ncand, int grid_points, double maxq,
                                                              double* __restrict__ cand_s, double* __restrict__ cand_z) {
    const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const double* w = Wk + (long long)row * ldw + c0;
    double lo = 0.0, hi = 0.0;
    for (int c = lane; c < ncols; c += 64) { const double v = w[c]; lo = fmin(lo, v); hi = fmax(hi, v); }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { lo = fmin(lo, __shfl_xor(lo, o, 64)); hi = fmax(hi, __shfl_xor(hi, o, 64)); }
    if (lo == hi) { lo = -1.0; hi = 1.0; }
    for (int k = lane; k < ncand; k += 64) {
        const double p = 1.0 - (double)k / (double)grid_points;
        const double s = (p * hi - p * lo) / maxq;
        const double z = rint(-(p * lo) / s);
        cand_s[(long long)row * ncand + k] = s;
        cand_z[(long long)row * ncand + k] = z;
    }
}

// Delta[(row, k), c] = s_k (clamp(round(w_c / s_k) + z_k) - z_k) - w_c
__global__ __launch_bounds__(256) void grid_delta_kernel(const double* __restrict__ Wk, long long ldw, int c0, int ncols, int ncand,
                                                         double maxq, const double* __restrict__ cand_s,
                                                         const double* __restrict__ cand_z, double* __restrict__ Delta) {
    const int row = blockIdx.y;
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= ncols) return;
    const double w = Wk[(long long)row * ldw + c0 + c];
    const double* cs = cand_s + (long long)row * ncand;
    const double* cz = cand_z + (long long)row * ncand;
    double* out = Delta + (long long)row * ncand * ncols + c;
    for (int k = 0; k < ncand; ++k) {
        const double s = cs[k], z = cz[k];
        const double q = quant_code(w, s, z, maxq);
        out[(long long)k * ncols] = s * (q - z) - w;
    }
}

// out[i] = sum_c A[i, c] B[i, c], one wavefront per row
__global__ __launch_bounds__(256) void rowdot_kernel(const double* __restrict__ A, long long lda, const double* __restrict__ B,
                                                     long long ldb, long long rows, int ncols, double* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const double* a = A + row * lda; const double* b = B + row * ldb;
    double s = 0.0;
    for (int c = lane; c < ncols; c += 64) s += a[c] * b[c];
    s = wave_sum(s);
    if (lane == 0) out[row] = s;
}

// lowest k among the minima of cost[row, :] -> (s, z) of that candidate
__global__ void grid_argmin_kernel(const double* __restrict__ cost, const double* __restrict__ cand_s,
                                   const double* __restrict__ cand_z, int rows, int ncand, BlockMap m, int r_off,
                                   double* __restrict__ s_out, double* __restrict__ z_out, int ng, int gi) {
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    const double* c = cost + (long long)row * ncand;
    int best = 0; double bc = c[0];
    for (int k = 1; k < ncand; ++k) if (c[k] < bc) { bc = c[k]; best = k; }
    const long long lr = layer_row(m, r_off + row);
    s_out[lr * ng + gi] = cand_s[(long long)row * ncand + best];
    z_out[lr * ng + gi] = cand_z[(long long)row * ncand + best];
}

// ---- two-phase search: approximate costs of all candidates on the bf16 matrix cores, exact fp64 costs of the few
// candidates within GRID_TAU of the approximate minimum.  delta and H_in are each split into an exact-to-16-bits (hi, lo)
// bf16 pair and  delta H  ~  hi.hi + lo.hi + hi.lo  is one GEMM over three concatenated segments.  Both need their second
// term: the cost is a difference of large terms when the input channels are correlated (cost / (|delta| |H| |delta|^T)
// of 2e-3 is ordinary), so an operand carried to 8 bits leaves errors of 1e-2 of the cost, five times GRID_TAU, and the
// true minimum can fall outside the survivors; with 16 bits on both sides the error is some 1e-5 of the cost.  As a guard,
// every exact re-evaluation is compared with its approximation, and a pass whose largest deviation exceeds a quarter of
// GRID_TAU is repeated with exact costs for every candidate (counted by tboa_counter).
constexpr int GRID_PAD = 256;        // extra elements per row of the concatenated operands (memory-channel spread)
constexpr int GRID_KS = 6;          // exact re-evaluations per row
constexpr double GRID_TAU = 2e-3;   // survivors: approximate cost <= (1 + tau) * approximate minimum

typedef __hip_bfloat16 bf16;

constexpr int GRID_TERMS = 3;        // segments of the concatenated contraction axis: [hi | lo | hi] of delta against [hi | hi | lo] of T

// H_in is symmetric, so delta H delta^T = 2 delta T delta^T with T = the lower triangle of H and half its diagonal: the GEMM
// then needs, for output column r, only the contraction indices c <= r (its causal limit), half the products.
// Hcat[b, r, :] = [hi(T[r,:]) | hi(T[r,:]) | lo(T[r,:])]; blocked: every [n, 3n + pad] matrix in the 16 x 32 blocks of the bf16 GEMM
__global__ void hcat_kernel(const double* __restrict__ H, bf16* __restrict__ out, int n, long long total, int blocked) {
    const long long pitch = GRID_TERMS * n + GRID_PAD;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const long long row = i / n; const int c = (int)(i % n);
        const int rr = (int)(row % n);
        const float v = c < rr ? (float)H[i] : c == rr ? (float)(0.5 * H[i]) : 0.f;
        const bf16 hi = __float2bfloat16(v), lo = __float2bfloat16(v - __bfloat162float(hi));
        if (blocked) {
            bf16* o = out + (row / n) * n * pitch; const long long r = row % n;
            o[tboa_blocked_offset(r, c, pitch >> 5)] = hi; o[tboa_blocked_offset(r, n + c, pitch >> 5)] = hi;
            o[tboa_blocked_offset(r, 2 * n + c, pitch >> 5)] = lo;
        } else {
            bf16* o = out + row * pitch + c;
            o[0] = hi; o[n] = hi; o[2 * n] = lo;
        }
    }
}

// Acat[(row, k), :] = [hi(delta) | lo(delta) | hi(delta)], delta as in grid_delta_kernel; mat_rows > 0: Acat is a sequence of matrices
// of mat_rows rows each (the rows that share one H_in), every one kept in the 16 x 32 blocks of the bf16 GEMM
__global__ __launch_bounds__(256) void grid_delta_split_kernel(const double* __restrict__ Wk, long long ldw, int n, int ncand, double maxq,
                                                               const double* __restrict__ cand_s, const double* __restrict__ cand_z,
                                                               bf16* __restrict__ Acat, long long mat_rows) {
    // four consecutive columns per thread (they share a 16-byte chunk of a block): 8-byte stores
    const int row = blockIdx.y;
    const int c = 4 * (blockIdx.x * blockDim.x + threadIdx.x);
    if (c >= n) return;
    const int nv = n - c < 4 ? n - c : 4;
    const bool vec = nv == 4 && n % 4 == 0;
    double w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = j < nv ? Wk[(long long)row * ldw + c + j] : 0.0;
    const double* cs = cand_s + (long long)row * ncand;
    const double* cz = cand_z + (long long)row * ncand;
    const long long pitch = (long long)GRID_TERMS * n + GRID_PAD;
    for (int k = 0; k < ncand; ++k) {
        const double s = cs[k], z = cz[k];
        union { bf16 b[4]; uint2 u; } hi, lo;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float dl = (float)(s * (quant_code(w[j], s, z, maxq) - z) - w[j]);
            hi.b[j] = __float2bfloat16(dl); lo.b[j] = __float2bfloat16(dl - __bfloat162float(hi.b[j]));
        }
        const long long R = (long long)row * ncand + k;
        bf16* o; long long o0, o1, o2;
        if (mat_rows > 0) {
            o = Acat + (R / mat_rows) * mat_rows * pitch; const long long r = R % mat_rows;
            o0 = tboa_blocked_offset(r, c, pitch >> 5); o1 = tboa_blocked_offset(r, n + c, pitch >> 5); o2 = tboa_blocked_offset(r, 2 * n + c, pitch >> 5);
        } else { o = Acat + R * pitch; o0 = c; o1 = n + c; o2 = 2 * n + c; }
        if (vec) { *(uint2*)(o + o0) = hi.u; *(uint2*)(o + o1) = lo.u; *(uint2*)(o + o2) = hi.u; }
        else
            for (int j = 0; j < nv; ++j) {     // (a blocked Acat has n % 32 == 0 and never comes here)
                o[o0 + j] = hi.b[j]; o[o1 + j] = lo.b[j]; o[o2 + j] = hi.b[j];
            }
    }
}

// cost[i] = 2 sum_c G[i, c] (hi + lo)[i, c], one wavefront per row (G = delta T^T, see hcat_kernel)
__global__ __launch_bounds__(256) void rowdot_split_kernel(const float* __restrict__ G, const bf16* __restrict__ Acat, long long rows, int n,
                                                           double* __restrict__ out, long long mat_rows) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const long long pitch = (long long)GRID_TERMS * n + GRID_PAD;
    const float* g = G + row * n; const bf16* a = Acat + row * pitch;
    double s = 0.0;
    if (n % 4 == 0) {     // four consecutive columns per lane (they share a 16-byte chunk of a block): 16- and 8-byte streaming loads
        typedef float f4 __attribute__((ext_vector_type(4)));
        const bf16* base = mat_rows > 0 ? Acat + (row / mat_rows) * mat_rows * pitch : a;
        const long long r = mat_rows > 0 ? row % mat_rows : 0;
        for (int c = 4 * lane; c < n; c += 256) {
            const f4 gv = __builtin_nontemporal_load((const f4*)(g + c));
            union { uint2 u; bf16 b[4]; } hi, lo;
            if (mat_rows > 0) {
                hi.u = *(const uint2*)(base + tboa_blocked_offset(r, c, pitch >> 5));
                lo.u = *(const uint2*)(base + tboa_blocked_offset(r, n + c, pitch >> 5));
            } else { hi.u = *(const uint2*)(a + c); lo.u = *(const uint2*)(a + n + c); }
#pragma unroll
            for (int j = 0; j < 4; ++j) s += (double)gv[j] * ((double)__bfloat162float(hi.b[j]) + (double)__bfloat162float(lo.b[j]));
        }
    } else if (mat_rows > 0) {
        a = Acat + (row / mat_rows) * mat_rows * pitch; const long long r = row % mat_rows;
        for (int c = lane; c < n; c += 64)
            s += (double)g[c] * ((double)__bfloat162float(a[tboa_blocked_offset(r, c, pitch >> 5)]) +
                                 (double)__bfloat162float(a[tboa_blocked_offset(r, n + c, pitch >> 5)]));
    } else
    for (int c = lane; c < n; c += 64) s += (double)g[c] * ((double)__bfloat162float(a[c]) + (double)__bfloat162float(a[n + c]));
    s = wave_sum(s);
    if (lane == 0) out[row] = 2.0 * s;
}

// Device-side bookkeeping of the two-phase search, accumulated over every pass of a quantize_layer call and read once at
// its end: [0] set when a pass could not be trusted as it stands (non-finite approximate cost, more near-minimal
// candidates in a group of rows than the exact re-evaluation has room for), [1] near-minimal candidates evaluated exactly,
// [2] the largest |approximate - exact| / |exact| seen, as the bits of a non-negative float.
enum { GS_TRIPPED = 0, GS_SURVIVORS = 1, GS_MAXDEV = 2, GS_WORDS = 3 };

// per row: the limit below which a candidate's approximate cost makes it a survivor, and the number of survivors that the
// exact pass evaluates.  A row with a single survivor needs none (that candidate wins), except every eighth row, whose
// exact cost is what the deviation guard of the pass measures.
__global__ void grid_count_kernel(const double* __restrict__ cost, int rows, int ncand, double tau, double* __restrict__ lim_out,
                                  int* __restrict__ cnt_out, int* __restrict__ gstat) {
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    const double* c = cost + (long long)row * ncand;
    double m = c[0];
    bool bad = !(c[0] == c[0]);
    for (int k = 1; k < ncand; ++k) { m = fmin(m, c[k]); bad |= !(c[k] == c[k]); }
    const double lim = m + tau * fabs(m);
    int cnt = 0;
    for (int k = 0; k < ncand; ++k) cnt += (c[k] <= lim) ? 1 : 0;
    if (bad || !(m == m) || cnt == 0) { atomicOr(gstat + GS_TRIPPED, 1); cnt = 0; }
    lim_out[row] = lim;
    const int ev = (cnt > 1 || row % 8 == 0) ? cnt : 0;
    cnt_out[row] = ev;
    if (ev) atomicAdd(gstat + GS_SURVIVORS, ev);
}

// exclusive prefix sums of cnt over the rows of each group of `per` rows (one workgroup per group): off[row], total[group];
// a group with more survivors than `cap` slots trips the guard, and its total is cut to cap (rows beyond are not evaluated)
__global__ __launch_bounds__(256) void grid_scan_kernel(const int* __restrict__ cnt, int per, int cap, int* __restrict__ off,
                                                        int* __restrict__ total, int* __restrict__ gstat) {
    __shared__ int part[256];
    const int g = blockIdx.x, t = threadIdx.x;
    const int* c = cnt + (long long)g * per; int* o = off + (long long)g * per;
    const int chunk = (per + 255) / 256, lo = t * chunk, hi = min(per, lo + chunk);
    int s = 0;
    for (int i = lo; i < hi; ++i) s += c[i];
    part[t] = s;
    __syncthreads();
    if (t == 0) {
        int run = 0;
        for (int i = 0; i < 256; ++i) { const int v = part[i]; part[i] = run; run += v; }
        if (run > cap) { atomicOr(gstat + GS_TRIPPED, 1); run = cap; }
        total[g] = run;
    }
    __syncthreads();
    int run = part[t];
    for (int i = lo; i < hi; ++i) { o[i] = run; run += c[i]; }
}

// exact delta of the survivors, compacted per group of `per` rows: DeltaS[group][off[row] + j, c] for the j-th survivor of
// the row (increasing k); slots at or beyond cap do not exist
__global__ __launch_bounds__(256) void grid_delta_sel_kernel(const double* __restrict__ Wk, long long ldw, int n, int ncand, double maxq,
                                                             const double* __restrict__ cand_s, const double* __restrict__ cand_z,
                                                             const double* __restrict__ cost, const double* __restrict__ lim,
                                                             const int* __restrict__ cnt, const int* __restrict__ off,
                                                             int per, int cap, double* __restrict__ DeltaS) {
    const int row = blockIdx.y;
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= n || cnt[row] == 0) return;
    const double w = Wk[(long long)row * ldw + c];
    const double l = lim[row];
    const double* cr = cost + (long long)row * ncand;
    double* out = DeltaS + ((long long)(row / per) * cap) * n + c;
    int slot = off[row];
    for (int k = 0; k < ncand && slot < cap; ++k) {
        if (!(cr[k] <= l)) continue;
        const double s = cand_s[(long long)row * ncand + k], z = cand_z[(long long)row * ncand + k];
        out[(long long)slot * n] = s * (quant_code(w, s, z, maxq) - z) - w;
        ++slot;
    }
}

// cost[i] = sum_c A[i, c] B[i, c] for the compacted rows: row i of group g (`slots` each) exists if i < total[g]
__global__ __launch_bounds__(256) void rowdot_limited_kernel(const double* __restrict__ A, const double* __restrict__ B, int n, int slots,
                                                             long long rows, const int* __restrict__ total, double* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    if ((int)(row % slots) >= total[row / slots]) return;
    const double* a = A + row * n; const double* b = B + row * n;
    double s = 0.0;
    for (int c = lane; c < n; c += 64) s += a[c] * b[c];
    s = wave_sum(s);
    if (lane == 0) out[row] = s;
}

// lowest exact cost among the survivors of a row (lowest k among equals: they are visited in increasing k); a row whose
// survivors were not evaluated takes its first one (it has a single one, or the pass is void anyway).  Every exact
// re-evaluation is compared with its approximation for the guard.
__global__ void grid_argmin_sel_kernel(const double* __restrict__ costS, const double* __restrict__ cost, const double* __restrict__ lim,
                                       const int* __restrict__ cnt, const int* __restrict__ off, int per, int cap,
                                       const double* __restrict__ cand_s, const double* __restrict__ cand_z, int rows, int ncand,
                                       BlockMap m, int r_off, double* __restrict__ s_out, double* __restrict__ z_out, int ng, int gi,
                                       int* __restrict__ gstat) {
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    const double* cr = cost + (long long)row * ncand;
    const double l = lim[row];
    const int nc = cnt[row];
    int best = -1;
    if (nc > 0) {
        const double* ce = costS + (long long)(row / per) * cap;
        int slot = off[row];
        double bc = 0.0, dev = 0.0;
        for (int k = 0; k < ncand && slot < cap; ++k) {
            if (!(cr[k] <= l)) continue;
            const double e = ce[slot];
            if (best < 0 || e < bc) { bc = e; best = k; }
            const double d = fabs(cr[k] - e) / fabs(e);
            dev = (d == d) ? fmax(dev, d) : 1.0;
            ++slot;
        }
        atomicMax(gstat + GS_MAXDEV, __float_as_int((float)fmin(dev, 1.0)));
    }
    if (best < 0) {
        best = 0;
        for (int k = 0; k < ncand; ++k) if (cr[k] <= l) { best = k; break; }
    }
    const long long lr = layer_row(m, r_off + row);
    s_out[lr * ng + gi] = cand_s[(long long)row * ncand + best];
    z_out[lr * ng + gi] = cand_z[(long long)row * ncand + best];
}

__global__ void clear_words_kernel(int* p, int n) { if ((int)threadIdx.x < n) p[threadIdx.x] = 0; }

// ------------------------------------------------------------------------------------------------ Algorithm 3
constexpr int SWEEP_SP = 512;      // columns whose updates of the columns further right are applied in one product
struct SweepArgs {
    double* Wk; int n; int nbr; BlockMap map;
    const double* U; const double* P; int per_head;   // U, P: [n, n] or [n_heads, n, n]
    int c0, pw;
    const double* s; const double* z; int ng, gi; double maxq;
    uint8_t* codes; double* Q;       // layer arrays [d_out, n]
    double* Epan; double* Wsnap;     // block arrays [rows, epitch], already offset to this panel's first column
    int epitch;
};

template <int RPW>
__global__ __launch_bounds__(256) void sweep_panel_kernel(SweepArgs a) {
    __shared__ double Us[64][64];
    __shared__ double Ps[64][64];
    const int h = blockIdx.y, n = a.n, c0 = a.c0, pw = a.pw;
    const double* U = a.U + (a.per_head ? (long long)h * n * n : 0);
    const double* P = a.P ? a.P + (a.per_head ? (long long)h * n * n : 0) : nullptr;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int j = i >> 6, k = i & 63;
        const bool in = (j < pw && k < pw);
        Us[j][k] = in ? U[(long long)(c0 + j) * n + c0 + k] : 0.0;
        Ps[j][k] = (in && P) ? P[(long long)(c0 + j) * n + c0 + k] : 0.0;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double w[RPW], s[RPW], z[RPW], qv[RPW], Qv[RPW], ev[RPW], wsv[RPW];
    int R[RPW]; bool valid[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        const int r = (blockIdx.x * 4 + wave) * RPW + i;
        valid[i] = r < a.nbr;
        R[i] = h * a.nbr + (valid[i] ? r : 0);
        const long long lr = layer_row(a.map, R[i]);
        w[i] = (valid[i] && lane < pw) ? a.Wk[(long long)R[i] * n + c0 + lane] : 0.0;
        s[i] = a.s[lr * a.ng + a.gi]; z[i] = a.z[lr * a.ng + a.gi];
        qv[i] = Qv[i] = ev[i] = wsv[i] = 0.0;
    }
    const bool hasP = (P != nullptr);
    for (int j = 0; j < pw; ++j) {
        const double urow = Us[j][lane], prow = Ps[j][lane], ujj = Us[j][j];
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const double wj = readlane_f64(w[i], j);
            const double q = quant_code(wj, s[i], z[i], a.maxq);
            const double Qj = s[i] * (q - z[i]);
            const double e = (wj - Qj) / ujj;
            if (lane == j) { qv[i] = q; Qv[i] = Qj; ev[i] = e; wsv[i] = wj; }
            w[i] = w[i] - e * urow;
            if (hasP) w[i] = w[i] - wj * prow;
        }
    }
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        if (!valid[i]) continue;
        if (lane < pw) {
            a.Epan[(long long)R[i] * a.epitch + lane] = ev[i];
            a.Wsnap[(long long)R[i] * a.epitch + lane] = wsv[i];
            const long long lr = layer_row(a.map, R[i]);
            a.codes[lr * n + c0 + lane] = (uint8_t)qv[i];
            a.Q[lr * n + c0 + lane] = Qv[i];
        }
    }
}

// ------------------------------------------------------------------------------------------------ Prop. 3.1 / 3.2
// E[R, c] = Wb[R, c] - Q[layer_row(R), c] (- S3[R, c])
__global__ void comp_error_kernel(const double* __restrict__ Wb, const double* __restrict__ Q, const double* __restrict__ S3,
                                  double* __restrict__ E, BlockMap m, int n) {
    const int R = blockIdx.y;
    const double* q = Q + layer_row(m, R) * n;
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n; c += gridDim.x * blockDim.x) {
        const long long i = (long long)R * n + c;
        double e = Wb[i] - q[c];
        if (S3) e -= S3[i];
        E[i] = e;
    }
}

// T[h, a, :] = Lo[a, B] Lo[B, B]^-1 for a = i1 .. dh-1, Lo = U_out[h]^T (lower): right-hand triangular solve,
// one thread per remaining row, columns from the last to the first.
__global__ void comp_T_kernel(const double* __restrict__ Uout, int dh, int i0, int i1, double* __restrict__ T, int TP) {
    const int h = blockIdx.y;
    const int a = i1 + blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= dh) return;
    const double* U = Uout + (long long)h * dh * dh;
    double* t = T + ((long long)h * dh + a) * TP;
    const int nb = i1 - i0;
    for (int c = nb - 1; c >= 0; --c) {
        double acc = U[(long long)(i0 + c) * dh + a];                 // Lo[a, i0+c]
        for (int k = c + 1; k < nb; ++k) acc -= t[k] * U[(long long)(i0 + c) * dh + i0 + k];   // Lo[i0+k, i0+c]
        t[c] = acc / U[(long long)(i0 + c) * dh + i0 + c];
    }
}

// ------------------------------------------------------------------------------------------------ Algorithm 2
// Wbar = codes - z (per group)
__global__ void wbar_kernel(const uint8_t* __restrict__ codes, const double* __restrict__ z, int ng, int gsz, int n,
                            double* __restrict__ Wbar) {
    const int r = blockIdx.y;
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n; c += gridDim.x * blockDim.x)
        Wbar[(long long)r * n + c] = (double)codes[(long long)r * n + c] - z[(long long)r * ng + c / gsz];
}

// Per head: s_j += sum_k (F[j,k] - s_k C[j,k]) Ho[k,j] / (C[j,j] Ho[j,j]) in order j = 0..dh-1,
// F = Wbar (W (H_in - R))^T, C = Wbar H_in Wbar^T   (Prop. 3.3 with Q = diag(s) Wbar)
__global__ __launch_bounds__(256) void cd_head_kernel(const double* __restrict__ F, const double* __restrict__ Cm,
                                                      const double* __restrict__ Ho, int dh, int iters, double* __restrict__ s_all) {
    extern __shared__ double sh[];
    double* s = sh; double* red = sh + dh;
    const int h = blockIdx.x, t = threadIdx.x;
    const double* Fh = F + (long long)h * dh * dh; const double* Ch = Cm + (long long)h * dh * dh;
    const double* Hh = Ho + (long long)h * dh * dh;
    double* sg = s_all + (long long)h * dh;
    for (int i = t; i < dh; i += 256) s[i] = sg[i];
    __syncthreads();
    for (int it = 0; it < iters; ++it)
        for (int j = 0; j < dh; ++j) {
            double acc = 0.0;
            for (int k = t; k < dh; k += 256) acc += (Fh[(long long)j * dh + k] - s[k] * Ch[(long long)j * dh + k]) * Hh[(long long)k * dh + j];
            acc = wave_sum(acc);
            if ((t & 63) == 0) red[t >> 6] = acc;
            __syncthreads();
            if (t == 0) {
                const double num = (red[0] + red[1]) + (red[2] + red[3]);
                const double den = Ch[(long long)j * dh + j] * Hh[(long long)j * dh + j];
                if (den > 0.0) s[j] = s[j] + num / den;
            }
            __syncthreads();
        }
    for (int i = t; i < dh; i += 256) sg[i] = s[i];
}

// Group-wise form of the same sweep: the coordinate is (row j, group g), visited in the order j = 0 .. dh-1,
// g = 0 .. ng-1, and Q = sum over (k, g') of s[k, g'] Wbar[k, G'] (rows masked to one group).  With
//   Cg[g][g'][j][k] = Wbar[j, G] H_in[G, G'] Wbar[k, G']^T      Fg[g][j][k] = Wbar[j, G] (W (H_in - R))[k, G]^T
// the step is  s[j, g] += sum_k Ho[k, j] (Fg[g][j][k] - sum_g' s[k, g'] Cg[g][g'][j][k]) / (Cg[g][g][j][j] Ho[j, j]).
// One workgroup per head; the scales of the head live in LDS.
__global__ __launch_bounds__(256) void cd_group_head_kernel(const double* __restrict__ Fg, const double* __restrict__ Cg,
                                                            const double* __restrict__ Ho, int dh, int ng, int iters,
                                                            double* __restrict__ s_all) {
    extern __shared__ double sh[];
    double* s = sh; double* hoj = sh + (size_t)dh * ng; double* red = hoj + dh;
    const int h = blockIdx.x, t = threadIdx.x;
    const long long rr = (long long)dh * dh;
    const double* Fh = Fg + (long long)h * ng * rr; const double* Ch = Cg + (long long)h * ng * ng * rr;
    const double* Hh = Ho + (long long)h * rr;
    double* sg = s_all + (long long)h * dh * ng;
    for (int i = t; i < dh * ng; i += 256) s[i] = sg[i];
    __syncthreads();
    for (int it = 0; it < iters; ++it)
        for (int j = 0; j < dh; ++j) {
            for (int k = t; k < dh; k += 256) hoj[k] = Hh[(long long)k * dh + j];
            __syncthreads();
            for (int g = 0; g < ng; ++g) {
                double acc = 0.0;
                for (int k = t; k < dh; k += 256) acc += Fh[((long long)g * dh + j) * dh + k] * hoj[k];
                for (int i = t; i < ng * dh; i += 256) {
                    const int g2 = i / dh, k = i - g2 * dh;
                    acc -= s[k * ng + g2] * Ch[(((long long)g * ng + g2) * dh + j) * dh + k] * hoj[k];
                }
                acc = wave_sum(acc);
                if ((t & 63) == 0) red[t >> 6] = acc;
                __syncthreads();
                if (t == 0) {
                    const double num = (red[0] + red[1]) + (red[2] + red[3]);
                    const double den = Ch[(((long long)g * ng + g) * dh + j) * dh + j] * hoj[j];
                    if (den > 0.0) s[j * ng + g] = s[j * ng + g] + num / den;
                }
                __syncthreads();
            }
        }
    for (int i = t; i < dh * ng; i += 256) sg[i] = s[i];
}

// out[row, seg] = sum over the columns c of segment seg of A[row, c] B[row, c]; one wavefront per (row, segment)
__global__ __launch_bounds__(256) void segdot_kernel(const double* __restrict__ A, const double* __restrict__ B, long long rows, int n, int gsz,
                                                     int ng, double* __restrict__ out, long long out_row_stride) {
    const int lane = threadIdx.x & 63;
    const long long w = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= rows * ng) return;
    const long long row = w / ng; const int seg = (int)(w - row * ng);
    const double* a = A + row * n + (long long)seg * gsz; const double* b = B + row * n + (long long)seg * gsz;
    double s = 0.0;
    for (int c = lane; c < gsz; c += 64) s += a[c] * b[c];
    s = wave_sum(s);
    if (lane == 0) out[row * out_row_stride + seg] = s;
}

// identity H_out with groups: per row, s[g] += (Fd[g] - sum_g' s[g'] Cd[g][g']) / Cd[g][g] in the order g = 0 .. ng-1.
// Cd [rows, ng, ng], Fd [rows, ng].  One wavefront per row, its scales in LDS.
__global__ __launch_bounds__(256) void cd_group_diag_kernel(const double* __restrict__ Fd, const double* __restrict__ Cd, long long rows, int ng,
                                                            int iters, double* __restrict__ s_all) {
    extern __shared__ double sh[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const long long row_raw = (long long)blockIdx.x * 4 + wv;
    const bool live = row_raw < rows;
    const long long row = live ? row_raw : rows - 1;
    double* s = sh + (size_t)wv * ng;
    for (int g = lane; g < ng; g += 64) s[g] = s_all[row * ng + g];
    __syncthreads();
    const double* C = Cd + row * ng * ng; const double* F = Fd + row * ng;
    for (int it = 0; it < iters; ++it)
        for (int g = 0; g < ng; ++g) {
            double acc = 0.0;
            for (int g2 = lane; g2 < ng; g2 += 64) acc += s[g2] * C[(long long)g * ng + g2];
            acc = wave_sum(acc);
            __syncthreads();
            if (lane == 0) { const double den = C[(long long)g * ng + g]; if (den > 0.0) s[g] = s[g] + (F[g] - acc) / den; }
            __syncthreads();
        }
    if (live) for (int g = lane; g < ng; g += 64) s_all[row * ng + g] = s[g];
}

// identity H_out: rows decouple, s_j += (F_jj - s_j C_jj) / C_jj
__global__ void cd_diag_kernel(const double* __restrict__ Fd, const double* __restrict__ Cd, int rows, int iters, double* __restrict__ s) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= rows) return;
    double v = s[j];
    for (int it = 0; it < iters; ++it) if (Cd[j] > 0.0) v = v + (Fd[j] - v * Cd[j]) / Cd[j];
    s[j] = v;
}

// Q = s * Wbar, plus the fp32 outputs
__global__ void finalize_kernel(const double* __restrict__ Wbar, const double* __restrict__ s, const double* __restrict__ z,
                                int ng, int gsz, int n, double* __restrict__ Q, float* __restrict__ Wdeq,
                                float* __restrict__ scales, float* __restrict__ zeros) {
    const int r = blockIdx.y;
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n; c += gridDim.x * blockDim.x) {
        const double q = s[(long long)r * ng + c / gsz] * Wbar[(long long)r * n + c];
        Q[(long long)r * n + c] = q;
        Wdeq[(long long)r * n + c] = (float)q;
    }
    if (blockIdx.x == 0)
        for (int g = threadIdx.x; g < ng; g += blockDim.x) {
            scales[(long long)r * ng + g] = (float)s[(long long)r * ng + g];
            zeros[(long long)r * ng + g] = (float)z[(long long)r * ng + g];
        }
}

// (Q - W) H_in from products that the scale refinement already formed, for one scale per row (Q = diag(s) Wbar):
// DH = diag(s) (Wbar H_in) - W H_in, with W H_in = Z + W R where Z = W (H_in - R).  Overwrites AH = Wbar H_in.
__global__ void dh_from_products_kernel(double* __restrict__ AH, const double* __restrict__ s, const double* __restrict__ Z,
                                        const double* __restrict__ WR, int n) {
    const int r = blockIdx.y;
    const double sr = s[r];
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n; c += gridDim.x * blockDim.x) {
        const long long i = (long long)r * n + c;
        const double wh = WR ? Z[i] + WR[i] : Z[i];
        AH[i] = sr * AH[i] - wh;
    }
}

// out[h] = scale * sum_{j,k} Ho[h][j,k] M[h][k,j]
__global__ __launch_bounds__(256) void head_trace_kernel(const double* __restrict__ Ho, const double* __restrict__ M, int dh,
                                                         double scale, double* __restrict__ out) {
    __shared__ double red[4];
    const int h = blockIdx.x, t = threadIdx.x;
    const double* Hh = Ho + (long long)h * dh * dh; const double* Mh = M + (long long)h * dh * dh;
    double acc = 0.0;
    for (int i = t; i < dh * dh; i += 256) { const int j = i / dh, k = i % dh; acc += Hh[i] * Mh[(long long)k * dh + j]; }
    acc = wave_sum(acc);
    if ((t & 63) == 0) red[t >> 6] = acc;
    __syncthreads();
    if (t == 0) out[h] = scale * ((red[0] + red[1]) + (red[2] + red[3]));
}

// out[h] = scale * sum over the rows of head h of v[row]
__global__ __launch_bounds__(256) void head_sum_kernel(const double* __restrict__ v, int dh, double scale, double* __restrict__ out) {
    __shared__ double red[4];
    const int h = blockIdx.x, t = threadIdx.x;
    double acc = 0.0;
    for (int i = t; i < dh; i += 256) acc += v[(long long)h * dh + i];
    acc = wave_sum(acc);
    if ((t & 63) == 0) red[t >> 6] = acc;
    __syncthreads();
    if (t == 0) out[h] = scale * ((red[0] + red[1]) + (red[2] + red[3]));
}

inline unsigned gx(long long n) { long long g = (n + 255) / 256; return (unsigned)(g < 1 ? 1 : (g > 64 ? 64 : g)); }

// ------------------------------------------------------------------------------------------------ host side
struct Layer {
    tboa_ctx* ctx; const tboa_layer_desc* d;
    int n, nh, dh, ng, gsz, nhin, ncand; double maxq;
    // workspace
    double *W64, *Wt, *Hi, *Hfac, *Uin, *Rd, *P, *Ho, *Hofac, *Uout, *ftmp, *fdinv;
    double *Q64, *s64, *z64;
    double *Wb, *Wk, *Epan, *Wsnap, *E, *S1, *S2, *T;
    double *cand_s, *cand_z, *Delta, *G, *cost, *DeltaS, *GS, *costS, *lim;
    __hip_bfloat16* Hcat; int* sel; int fast_grid, grid_blocked;
    double *Wbar, *Abar, *Z, *WR, *Cm, *Fm, *dvec, *lossbuf;
    double *Cg, *Fg;    // group-wise refinement: Gram blocks per (group, group) pair
    int grid_chunk;     // block rows (shared H_in) or heads (per-head H_in) per grid-search pass
    int* gstat;         // device words of the two-phase search (GS_*), cleared at the start of a run
    long long nn;
};

// Algorithm 1 line 9 for the rows Wrows (block rows of every head, or whole heads for the fixed grid), columns [c0, c0 + ncols).
// Everything is enqueued; nothing is read back here.
int grid_search(Layer& L, const double* Wrows, long long ldw, int rows_per_head, BlockMap map, int c0, int ncols, int gi) {
    tboa_ctx* ctx = L.ctx;
    const int nh = L.nh, ncand = L.ncand;
    const bool ph = L.nhin > 1;
    const int total_rows = nh * rows_per_head;
    const int units = ph ? nh : total_rows;                 // chunk unit: a head or a row
    const int rows_per_unit = ph ? rows_per_head : 1;
    for (int u0 = 0; u0 < units; u0 += L.grid_chunk) {
        const int nu = (units - u0 < L.grid_chunk) ? units - u0 : L.grid_chunk;
        const int r0 = u0 * rows_per_unit, rows = nu * rows_per_unit;
        const double* Wc = Wrows + (long long)r0 * ldw;
        hipLaunchKernelGGL(grid_candidates_kernel, dim3((rows + 3) / 4), dim3(256), 0, ctx->stream, Wc, ldw, c0, ncols, rows,
                           ncand, L.d->grid_points, L.maxq, L.cand_s, L.cand_z);
        TB_KERNEL_CHECK(ctx);
        if (L.fast_grid && c0 == 0 && ncols == L.n) {
            const int n = L.n;
            __hip_bfloat16* Acat = (__hip_bfloat16*)L.Delta; float* G32 = (float*)L.G;
            // both operands in the GEMM's 16 x 32 blocks when the shapes allow it (L.grid_blocked, decided with Hcat)
            long long mat_rows = L.grid_blocked ? (long long)(ph ? rows_per_head : rows) * ncand : 0;
            if (mat_rows % 16) mat_rows = 0;
            hipLaunchKernelGGL(grid_delta_split_kernel, dim3((n + 1023) / 1024, rows), dim3(256), 0, ctx->stream, Wc, ldw, n, ncand, L.maxq,
                               L.cand_s, L.cand_z, Acat, mat_rows);
            TB_KERNEL_CHECK(ctx);
            GemmBf16 a{};
            a.N = n; a.K = GRID_TERMS * n; a.alpha = 1.f; a.A = Acat; a.lda = (long long)GRID_TERMS * n + GRID_PAD; a.ldb = a.lda; a.C = G32; a.ldc = n;
            a.c_dtype = TBOA_F32; a.accumulate = 0; a.flags = (mat_rows > 0 ? TBOA_GEMM_A_TILED : 0) | (L.grid_blocked ? TBOA_GEMM_B_TILED : 0); a.tag = TBOA_PROF_GRID;
            a.flags |= TBOA_GEMM_CAUSAL_K; a.kseg = n;   // Hcat holds the lower triangle: contraction index <= output column, in every segment
            if (ph) { a.M = rows_per_head * ncand; a.batch = nu; a.B = L.Hcat + (long long)u0 * n * a.lda;
                      a.strideA = (long long)a.M * a.lda; a.strideB = (long long)n * a.lda; a.strideC = (long long)a.M * n; }
            else { a.M = rows * ncand; a.batch = 1; a.B = L.Hcat; }
            TB_TRY(gemm_bf16_nt(ctx, a));
            const long long crow = (long long)rows * ncand;
            hipLaunchKernelGGL(rowdot_split_kernel, dim3((unsigned)((crow + 3) / 4)), dim3(256), 0, ctx->stream, G32, Acat, crow, n, L.cost, mat_rows);
            const int per = ph ? rows_per_head : rows, ngrp = rows / per;    // rows that share one H_in
            const int cap = per * GRID_KS;                                    // exact re-evaluations a group has room for
            int* cntv = L.sel; int* offv = cntv + rows; int* totv = offv + rows;
            hipLaunchKernelGGL(grid_count_kernel, dim3((rows + 255) / 256), dim3(256), 0, ctx->stream, L.cost, rows, ncand, GRID_TAU, L.lim, cntv, L.gstat);
            hipLaunchKernelGGL(grid_scan_kernel, dim3(ngrp), dim3(256), 0, ctx->stream, cntv, per, cap, offv, totv, L.gstat);
            hipLaunchKernelGGL(grid_delta_sel_kernel, dim3((n + 255) / 256, rows), dim3(256), 0, ctx->stream, Wc, ldw, n, ncand, L.maxq,
                               L.cand_s, L.cand_z, L.cost, L.lim, cntv, offv, per, cap, L.DeltaS);
            TB_KERNEL_CHECK(ctx);
            GemmF64 g{};
            g.M = cap; g.N = n; g.K = n; g.alpha = 1.0; g.beta = 0.0; g.A = L.DeltaS; g.sam = n; g.sak = 1; g.sbk = n; g.sbn = 1;
            g.C = L.GS; g.ldc = n; g.batch = ngrp; g.strideA = (long long)g.M * n; g.strideC = g.strideA; g.m_limit = totv;
            g.B = L.Hi + (ph ? (long long)u0 * L.nn : 0); g.strideB = ph ? L.nn : 0;
            g.tag = TBOA_PROF_F64_GRID;
            TB_TRY(gemm_f64(ctx, g));
            const long long srow = (long long)ngrp * cap;
            hipLaunchKernelGGL(rowdot_limited_kernel, dim3((unsigned)((srow + 3) / 4)), dim3(256), 0, ctx->stream, L.GS, L.DeltaS, n, cap,
                               srow, totv, L.costS);
            hipLaunchKernelGGL(grid_argmin_sel_kernel, dim3((rows + 255) / 256), dim3(256), 0, ctx->stream, L.costS, L.cost, L.lim, cntv, offv, per, cap,
                               L.cand_s, L.cand_z, rows, ncand, map, r0, L.s64, L.z64, L.ng, gi, L.gstat);
            TB_KERNEL_CHECK(ctx);
            ++ctx->counters[TBOA_CTR_GRID_PASSES];
            continue;
        }
        hipLaunchKernelGGL(grid_delta_kernel, dim3((ncols + 255) / 256, rows), dim3(256), 0, ctx->stream, Wc, ldw, c0, ncols, ncand,
                           L.maxq, L.cand_s, L.cand_z, L.Delta);
        TB_KERNEL_CHECK(ctx);
        GemmF64 g{};
        g.N = ncols; g.K = ncols; g.alpha = 1.0; g.beta = 0.0;
        g.A = L.Delta; g.sam = ncols; g.sak = 1;
        g.sbk = L.n; g.sbn = 1; g.C = L.G; g.ldc = ncols;
        g.tag = TBOA_PROF_F64_GRID;
        if (ph) {
            g.M = rows_per_head * ncand; g.batch = nu;
            g.B = L.Hi + (long long)u0 * L.nn + (long long)c0 * L.n + c0;
            g.strideA = (long long)g.M * ncols; g.strideB = L.nn; g.strideC = g.strideA;
        } else {
            g.M = rows * ncand; g.batch = 1;
            g.B = L.Hi + (long long)c0 * L.n + c0;
        }
        TB_TRY(gemm_f64(ctx, g));
        const long long crow = (long long)rows * ncand;
        hipLaunchKernelGGL(rowdot_kernel, dim3((unsigned)((crow + 3) / 4)), dim3(256), 0, ctx->stream, L.G, (long long)ncols, L.Delta,
                           (long long)ncols, crow, ncols, L.cost);
        hipLaunchKernelGGL(grid_argmin_kernel, dim3((rows + 255) / 256), dim3(256), 0, ctx->stream, L.cost, L.cand_s, L.cand_z, rows,
                           ncand, map, r0, L.s64, L.z64, L.ng, gi);
        TB_KERNEL_CHECK(ctx);
    }
    return 0;
}

// one GEMM over all block rows (shared H_in) or batched per head (per-head H_in): C = alpha A op(B) + beta C,
// A, C block arrays [nh*nbr, *]; B a d_in x d_in matrix (or one per head) addressed by (sbk, sbn) at offset boff.
int block_gemm(Layer& L, int nbr, int N, int K, double alpha, const double* A, long long lda, const double* B, long long boff,
               long long sbk, long long sbn, double beta, double* C, long long ldc, int tag, const GemmF64* flags = nullptr) {
    GemmF64 g{};
    if (flags) g = *flags;
    g.tag = tag;
    g.N = N; g.K = K; g.alpha = alpha; g.beta = beta;
    g.A = A; g.sam = lda; g.sak = 1; g.B = B + boff; g.sbk = sbk; g.sbn = sbn; g.C = C; g.ldc = ldc;
    if (L.nhin > 1) { g.M = nbr; g.batch = L.nh; g.strideA = (long long)nbr * lda; g.strideB = L.nn; g.strideC = (long long)nbr * ldc; }
    else { g.M = L.nh * nbr; g.batch = 1; }
    return gemm_f64(L.ctx, g);
}

// return value of run_layer: the approximate costs of the two-phase grid search could not be trusted somewhere in this
// run (see grid_search): the caller runs the layer again with exact costs for every candidate
constexpr int RUN_AGAIN_EXACT = 1;

int run_layer(Layer& L, const void* W, const float* H_in, const float* H_out, const float* R, uint8_t* codes, float* scales,
              float* zeros, float* W_deq, double* loss, double* loss_per_head) {
    tboa_ctx* ctx = L.ctx; const tboa_layer_desc* d = L.d;
    const int n = L.n, nh = L.nh, dh = L.dh, ng = L.ng, nhin = L.nhin;
    const long long nn = L.nn, wn = (long long)d->d_out * n;
    hipStream_t st = ctx->stream;

    hipLaunchKernelGGL(clear_words_kernel, dim3(1), dim3(64), 0, st, L.gstat, (int)GS_WORDS);
    TB_KERNEL_CHECK(ctx);

    TB_TRY(launch_cvt_to_f64(ctx, W, d->w_dtype, L.W64, wn));
    TB_HIP(ctx, hipMemcpyAsync(L.Wt, L.W64, wn * sizeof(double), hipMemcpyDeviceToDevice, st));
    // eq. 3 for H_in (and H_out)
    TB_TRY(launch_f32_to_f64_damp(ctx, n, nhin, H_in, d->damp, L.Hi));
    TB_HIP(ctx, hipMemcpyAsync(L.Hfac, L.Hi, nhin * nn * sizeof(double), hipMemcpyDeviceToDevice, st));
    if (L.fast_grid) {
        long long tot = nhin * nn, gb = (tot + 255) / 256; if (gb > 32768) gb = 32768;
        hipLaunchKernelGGL(hcat_kernel, dim3((unsigned)gb), dim3(256), 0, st, L.Hi, L.Hcat, n, tot, L.grid_blocked);
        TB_KERNEL_CHECK(ctx);
    }
    // U_in, P and U_out are first needed by the first in-channel sweep; the grid search before it needs only W and H_in.
    // The factorisations and the two P products (for one matrix: chains of small kernels that leave most of the GPU idle)
    // therefore run on the context's second stream, beside that grid search; setup_join() below is where they meet.
    // The breakdown status of the factorisations is read at the end of the call, with everything else that comes back.
    struct StreamSwap {      // everything enqueued while this lives goes to the second stream
        tboa_ctx* c; hipStream_t keep;
        explicit StreamSwap(tboa_ctx* c_) : c(c_), keep(c_->stream) { c->stream = c->aux; }
        ~StreamSwap() { c->stream = keep; }
    };
    bool joined = false;
    struct DrainAux {      // an error return before the join must not leave work running on the workspace
        tboa_ctx* c; const bool* joined;
        ~DrainAux() { if (!*joined) (void)hipStreamSynchronize(c->aux); }
    } drain{ctx, &joined};
    TB_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
    {
    StreamSwap swap(ctx);
    TB_HIP(ctx, hipStreamWaitEvent(ctx->aux, ctx->ev_fork, 0));
    TB_TRY(chol_inv_upper_f64(ctx, n, nhin, L.Hfac, L.Uin, L.ftmp, L.fdinv, 0, true));
    if (R) {   // Algorithm 3 line 2: P = ((R U^T) * M_U) U
        TB_TRY(launch_cvt_f32_to_f64(ctx, R, L.Rd, nhin * nn));
        GemmF64 a{};
        a.M = n; a.N = n; a.K = n; a.alpha = 1.0; a.beta = 0.0;
        a.A = L.Rd; a.sam = n; a.sak = 1; a.B = L.Uin; a.sbk = 1; a.sbn = n; a.klo_n = 1;   // U[c, k] = 0 for k < c
        a.skip_lower = 1;   // only the part above the diagonal survives the mask below
        a.C = L.Hfac; a.ldc = n; a.batch = nhin; a.strideA = nn; a.strideB = nn; a.strideC = nn;
        a.tag = TBOA_PROF_F64_FACTOR;
        TB_TRY(gemm_f64(ctx, a));
        TB_TRY(launch_strict_upper_f64(ctx, L.Hfac, n, nhin));
        GemmF64 b{};
        b.M = n; b.N = n; b.K = n; b.alpha = 1.0; b.beta = 0.0;
        b.A = L.Hfac; b.sam = n; b.sak = 1; b.klo_m = 1;       // (R U^T)_masked[j, m] = 0 for m <= j
        b.B = L.Uin; b.sbk = n; b.sbn = 1; b.khi_n = 1;        // U[m, k] = 0 for m > k
        b.diag_order = 1;                                      // contraction range (row start, column end]: grows with the column
        b.C = L.P; b.ldc = n; b.batch = nhin; b.strideA = nn; b.strideB = nn; b.strideC = nn;
        b.tag = TBOA_PROF_F64_FACTOR;
        TB_TRY(gemm_f64(ctx, b));
    }
    if (H_out) {
        TB_TRY(launch_f32_to_f64_damp(ctx, dh, nh, H_out, d->damp, L.Ho));
        TB_HIP(ctx, hipMemcpyAsync(L.Hofac, L.Ho, (size_t)nh * dh * dh * sizeof(double), hipMemcpyDeviceToDevice, ctx->stream));
        TB_TRY(chol_inv_upper_f64(ctx, dh, nh, L.Hofac, L.Uout, L.ftmp, L.fdinv, 2, true));
    }
    TB_HIP(ctx, hipEventRecord(ctx->ev_join, ctx->aux));
    }
    auto setup_join = [&]() -> int {
        if (joined) return 0;
        TB_HIP(ctx, hipStreamWaitEvent(st, ctx->ev_join, 0));
        joined = true;
        return 0;
    };
    const double* Pp = R ? L.P : nullptr;
    const int pw_max = L.gsz < 64 ? L.gsz : 64;
    // columns per group of panels: a group-wise grid is searched on the current columns of its group when the sweep enters
    // it, so a group of panels must not straddle a grid group that starts inside it unaligned
    const int sp = (!d->group || SWEEP_SP % L.gsz == 0 || L.gsz % SWEEP_SP == 0) ? SWEEP_SP : pw_max;

    if (!d->adaptive_grid) {   // BoA: one grid from the original weights
        BlockMap id{dh, dh, 0};
        for (int gi = 0; gi < ng; ++gi) TB_TRY(grid_search(L, L.W64, n, dh, id, gi * L.gsz, L.gsz, gi));
    }
    for (int i0 = 0; i0 < dh; i0 += d->block) {
        const int i1 = (i0 + d->block < dh) ? i0 + d->block : dh;
        const int nbr = i1 - i0, rows = nh * nbr;
        BlockMap map{nbr, dh, i0};
        hipLaunchKernelGGL(gather_rows_kernel, dim3(gx(n), rows), dim3(256), 0, st, L.Wt, L.Wb, map, n);
        TB_KERNEL_CHECK(ctx);
        TB_HIP(ctx, hipMemcpyAsync(L.Wk, L.Wb, (size_t)rows * n * sizeof(double), hipMemcpyDeviceToDevice, st));
        if (d->adaptive_grid && !d->group) TB_TRY(grid_search(L, L.Wk, n, nbr, map, 0, n, 0));
        // Algorithm 3 in panels on two levels: inside a group of up to SWEEP_SP columns every 64-column panel updates the rest of
        // the group at once; the columns right of the group get the group's whole update in one product (a contraction SWEEP_SP
        // deep instead of 64: a quarter of the passes over the remaining columns)
        for (int s0 = 0; s0 < n; s0 += sp) {
            const int s1 = (n - s0 < sp) ? n : s0 + sp;
            for (int c0 = s0; c0 < s1; c0 += pw_max) {
                const int pw = (s1 - c0 < pw_max) ? s1 - c0 : pw_max, c1 = c0 + pw;
                const int gi = c0 / L.gsz;
                if (d->group && d->adaptive_grid && c0 % L.gsz == 0) TB_TRY(grid_search(L, L.Wk, n, nbr, map, c0, L.gsz, gi));
                SweepArgs a;
                a.Wk = L.Wk; a.n = n; a.nbr = nbr; a.map = map; a.U = L.Uin; a.P = Pp; a.per_head = nhin > 1;
                a.c0 = c0; a.pw = pw; a.s = L.s64; a.z = L.z64; a.ng = ng; a.gi = gi; a.maxq = L.maxq;
                a.codes = codes; a.Q = L.Q64; a.Epan = L.Epan + (c0 - s0); a.Wsnap = L.Wsnap + (c0 - s0); a.epitch = SWEEP_SP;
                TB_TRY(setup_join());
                hipLaunchKernelGGL((sweep_panel_kernel<2>), dim3((nbr + 7) / 8, nh), dim3(256), 0, st, a);
                TB_KERNEL_CHECK(ctx);
                if (c1 < s1) {   // rest of the group: W[:, c1:s1] -= E U[c0:c1, c1:s1] + Wsnap P[c0:c1, c1:s1]
                    GemmF64 two{};   // both terms in one pass over the output
                    if (Pp) { two.A2 = L.Wsnap + (c0 - s0); two.B2 = L.P + (long long)c0 * n + c1; }
                    TB_TRY(block_gemm(L, nbr, s1 - c1, pw, -1.0, L.Epan + (c0 - s0), SWEEP_SP, L.Uin, (long long)c0 * n + c1, n, 1, 1.0, L.Wk + c1, n,
                                      TBOA_PROF_F64_SWEEP, &two));
                }
            }
            if (s1 < n) {   // columns right of the group: W[:, s1:] -= E U[s0:s1, s1:] + Wsnap P[s0:s1, s1:]
                GemmF64 two{};
                if (Pp) { two.A2 = L.Wsnap; two.B2 = L.P + (long long)s0 * n + s1; }
                TB_TRY(block_gemm(L, nbr, n - s1, s1 - s0, -1.0, L.Epan, SWEEP_SP, L.Uin, (long long)s0 * n + s1, n, 1, 1.0, L.Wk + s1, n,
                                  TBOA_PROF_F64_SWEEP, &two));
            }
        }
        if (H_out && i1 < dh) {
            const double* S3 = nullptr;
            if (R) {   // W_B R H_in^-1 = ((W_B R) U^T) U
                GemmF64 f1{}; f1.klo_n = 1;
                GemmF64 f2{}; f2.khi_n = 1;
                TB_TRY(block_gemm(L, nbr, n, n, 1.0, L.Wb, n, L.Rd, 0, n, 1, 0.0, L.S1, n, TBOA_PROF_F64_COMP));
                TB_TRY(block_gemm(L, nbr, n, n, 1.0, L.S1, n, L.Uin, 0, 1, n, 0.0, L.S2, n, TBOA_PROF_F64_COMP, &f1));
                TB_TRY(block_gemm(L, nbr, n, n, 1.0, L.S2, n, L.Uin, 0, n, 1, 0.0, L.S1, n, TBOA_PROF_F64_COMP, &f2));
                S3 = L.S1;
            }
            hipLaunchKernelGGL(comp_error_kernel, dim3(gx(n), rows), dim3(256), 0, st, L.Wb, L.Q64, S3, L.E, map, n);
            const int rem = dh - i1;
            hipLaunchKernelGGL(comp_T_kernel, dim3((rem + 63) / 64, nh), dim3(64), 0, st, L.Uout, dh, i0, i1, L.T, d->block);
            TB_KERNEL_CHECK(ctx);
            GemmF64 u{};   // W~[i1:, :] -= T E per head
            u.M = rem; u.N = n; u.K = nbr; u.alpha = -1.0; u.beta = 1.0;
            u.A = L.T + (long long)i1 * d->block; u.sam = d->block; u.sak = 1;
            u.B = L.E; u.sbk = n; u.sbn = 1;
            u.C = L.Wt + (long long)i1 * n; u.ldc = n;
            u.batch = nh; u.strideA = (long long)dh * d->block; u.strideB = (long long)nbr * n; u.strideC = (long long)dh * n;
            u.tag = TBOA_PROF_F64_COMP;
            TB_TRY(gemm_f64(ctx, u));
        }
    }

    // Algorithm 2 + outputs + loss
    const int rows_all = d->d_out;
    hipLaunchKernelGGL(wbar_kernel, dim3(gx(n), rows_all), dim3(256), 0, st, codes, L.z64, ng, L.gsz, n, L.Wbar);
    TB_KERNEL_CHECK(ctx);
    if (R) TB_TRY(block_gemm(L, dh, n, n, 1.0, L.W64, n, L.Rd, 0, n, 1, 0.0, L.WR, n, TBOA_PROF_F64_CD));
    if (d->cd_iters > 0 && d->group) {
        // Z = W (H_in - R); per group g: AH = Wbar[:, G] H_in[G, :] (into Abar), then the Gram blocks against every group
        const int gsz = L.gsz;
        const long long rr = (long long)dh * dh;
        TB_TRY(block_gemm(L, dh, n, n, 1.0, L.W64, n, L.Hi, 0, n, 1, 0.0, L.Z, n, TBOA_PROF_F64_CD));
        if (R) TB_TRY(launch_sub_f64(ctx, L.Z, L.WR, L.Z, wn));
        if (H_out) {
            GemmF64 f{};   // Fg[h][g] = Wbar_h[:, G] Z_h[:, G]^T
            f.M = dh; f.N = dh; f.K = gsz; f.alpha = 1.0; f.beta = 0.0;
            f.A = L.Wbar; f.sam = n; f.sak = 1; f.B = L.Z; f.sbk = 1; f.sbn = n; f.C = L.Fg; f.ldc = dh;
            f.batch = nh * ng; f.batch_inner = ng;
            f.strideA = (long long)dh * n; f.strideB = f.strideA; f.strideC = ng * rr;
            f.strideA2 = gsz; f.strideB2 = gsz; f.strideC2 = rr;
            TB_TRY(gemm_f64(ctx, f));
        } else {
            hipLaunchKernelGGL(segdot_kernel, dim3((unsigned)(((long long)rows_all * ng + 3) / 4)), dim3(256), 0, st, L.Wbar, L.Z,
                               (long long)rows_all, n, gsz, ng, L.Fg, (long long)ng);
            TB_KERNEL_CHECK(ctx);
        }
        for (int g = 0; g < ng; ++g) {
            TB_TRY(block_gemm(L, dh, n, gsz, 1.0, L.Wbar + (long long)g * gsz, n, L.Hi, (long long)g * gsz * n, n, 1, 0.0, L.Abar, n, TBOA_PROF_F64_CD));
            if (H_out) {
                GemmF64 c{};   // Cg[h][g][g'] = AH_h[:, G'] Wbar_h[:, G']^T
                c.M = dh; c.N = dh; c.K = gsz; c.alpha = 1.0; c.beta = 0.0;
                c.A = L.Abar; c.sam = n; c.sak = 1; c.B = L.Wbar; c.sbk = 1; c.sbn = n; c.C = L.Cg + (long long)g * ng * rr; c.ldc = dh;
                c.batch = nh * ng; c.batch_inner = ng;
                c.strideA = (long long)dh * n; c.strideB = c.strideA; c.strideC = (long long)ng * ng * rr;
                c.strideA2 = gsz; c.strideB2 = gsz; c.strideC2 = rr;
                TB_TRY(gemm_f64(ctx, c));
            } else {   // Cd[row][g][g'] = AH[row, G'] . Wbar[row, G']
                hipLaunchKernelGGL(segdot_kernel, dim3((unsigned)(((long long)rows_all * ng + 3) / 4)), dim3(256), 0, st, L.Abar, L.Wbar,
                                   (long long)rows_all, n, gsz, ng, L.Cg + (long long)g * ng, (long long)ng * ng);
                TB_KERNEL_CHECK(ctx);
            }
        }
        if (H_out) {
            const size_t smem = ((size_t)dh * ng + dh + 8) * sizeof(double);
            if (smem > 160 * 1024) return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: %d scales per head exceed the LDS of the group-wise refinement", dh * ng);
            TB_HIP(ctx, hipFuncSetAttribute((const void*)cd_group_head_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            hipLaunchKernelGGL(cd_group_head_kernel, dim3(nh), dim3(256), smem, st, L.Fg, L.Cg, L.Ho, dh, ng, d->cd_iters, L.s64);
        } else {
            const size_t smem = (size_t)4 * ng * sizeof(double);
            hipLaunchKernelGGL(cd_group_diag_kernel, dim3((rows_all + 3) / 4), dim3(256), smem, st, L.Fg, L.Cg, (long long)rows_all, ng,
                               d->cd_iters, L.s64);
        }
        TB_KERNEL_CHECK(ctx);
    } else if (d->cd_iters > 0) {
        TB_TRY(block_gemm(L, dh, n, n, 1.0, L.Wbar, n, L.Hi, 0, n, 1, 0.0, L.Abar, n, TBOA_PROF_F64_CD));
        TB_TRY(block_gemm(L, dh, n, n, 1.0, L.W64, n, L.Hi, 0, n, 1, 0.0, L.Z, n, TBOA_PROF_F64_CD));
        if (R) TB_TRY(launch_sub_f64(ctx, L.Z, L.WR, L.Z, wn));
        if (H_out) {
            GemmF64 c{};
            c.M = dh; c.N = dh; c.K = n; c.alpha = 1.0; c.beta = 0.0;
            c.A = L.Abar; c.sam = n; c.sak = 1; c.B = L.Wbar; c.sbk = 1; c.sbn = n; c.C = L.Cm; c.ldc = dh;
            c.batch = nh; c.strideA = (long long)dh * n; c.strideB = c.strideA; c.strideC = (long long)dh * dh;
            TB_TRY(gemm_f64(ctx, c));
            c.A = L.Wbar; c.B = L.Z; c.C = L.Fm;
            TB_TRY(gemm_f64(ctx, c));
            hipLaunchKernelGGL(cd_head_kernel, dim3(nh), dim3(256), (dh + 8) * sizeof(double), st, L.Fm, L.Cm, L.Ho, dh, d->cd_iters, L.s64);
        } else {
            hipLaunchKernelGGL(rowdot_kernel, dim3((rows_all + 3) / 4), dim3(256), 0, st, L.Abar, (long long)n, L.Wbar, (long long)n,
                               (long long)rows_all, n, L.dvec);
            hipLaunchKernelGGL(rowdot_kernel, dim3((rows_all + 3) / 4), dim3(256), 0, st, L.Wbar, (long long)n, L.Z, (long long)n,
                               (long long)rows_all, n, L.dvec + rows_all);
            hipLaunchKernelGGL(cd_diag_kernel, dim3((rows_all + 255) / 256), dim3(256), 0, st, L.dvec + rows_all, L.dvec, rows_all,
                               d->cd_iters, L.s64);
        }
        TB_KERNEL_CHECK(ctx);
    }
    hipLaunchKernelGGL(finalize_kernel, dim3(gx(n), rows_all), dim3(256), 0, st, L.Wbar, L.s64, L.z64, ng, L.gsz, n, L.Q64, W_deq,
                       scales, zeros);
    TB_KERNEL_CHECK(ctx);
    const bool want_loss = loss || loss_per_head;
    if (want_loss) {
        // D = Q - W (into Wbar), D H_in (into Abar)
        TB_TRY(launch_sub_f64(ctx, L.Q64, L.W64, L.Wbar, wn));
        if (d->cd_iters > 0 && !d->group) {   // Abar = Wbar H_in and Z are still those of the scale refinement
            hipLaunchKernelGGL(dh_from_products_kernel, dim3(gx(n), rows_all), dim3(256), 0, st, L.Abar, L.s64, L.Z, R ? L.WR : nullptr, n);
            TB_KERNEL_CHECK(ctx);
        } else TB_TRY(block_gemm(L, dh, n, n, 1.0, L.Wbar, n, L.Hi, 0, n, 1, 0.0, L.Abar, n, TBOA_PROF_F64_CD));
        double* lq = L.lossbuf; double* lc = L.lossbuf + nh;
        TB_TRY(launch_fill_f64(ctx, L.lossbuf, 2 * nh, 0.0));
        if (H_out) {
            GemmF64 c{};
            c.M = dh; c.N = dh; c.K = n; c.alpha = 1.0; c.beta = 0.0;
            c.A = L.Abar; c.sam = n; c.sak = 1; c.B = L.Wbar; c.sbk = 1; c.sbn = n; c.C = L.Cm; c.ldc = dh;
            c.batch = nh; c.strideA = (long long)dh * n; c.strideB = c.strideA; c.strideC = (long long)dh * dh;
            c.tag = TBOA_PROF_F64_CD;
            TB_TRY(gemm_f64(ctx, c));
            hipLaunchKernelGGL(head_trace_kernel, dim3(nh), dim3(256), 0, st, L.Ho, L.Cm, dh, 1.0, lq);
            if (R) {
                c.A = L.WR; c.B = L.Wbar; c.C = L.Fm;
                TB_TRY(gemm_f64(ctx, c));
                hipLaunchKernelGGL(head_trace_kernel, dim3(nh), dim3(256), 0, st, L.Ho, L.Fm, dh, 2.0, lc);
            }
        } else {
            hipLaunchKernelGGL(rowdot_kernel, dim3((rows_all + 3) / 4), dim3(256), 0, st, L.Abar, (long long)n, L.Wbar, (long long)n,
                               (long long)rows_all, n, L.dvec);
            hipLaunchKernelGGL(head_sum_kernel, dim3(nh), dim3(256), 0, st, L.dvec, dh, 1.0, lq);
            if (R) {
                hipLaunchKernelGGL(rowdot_kernel, dim3((rows_all + 3) / 4), dim3(256), 0, st, L.WR, (long long)n, L.Wbar, (long long)n,
                                   (long long)rows_all, n, L.dvec);
                hipLaunchKernelGGL(head_sum_kernel, dim3(nh), dim3(256), 0, st, L.dvec, dh, 2.0, lc);
            }
        }
        TB_KERNEL_CHECK(ctx);
    }
    // ---- the one place where the call waits for the device: factorisation status, the bookkeeping of the grid search, losses
    TB_TRY(setup_join());      // (a layer with no in-channel sweep at all never joined)
    double* host = nullptr;
    if (want_loss) {
        host = (double*)malloc(2 * (size_t)nh * sizeof(double));
        if (!host) return tboa_fail(ctx, TBOA_ENOMEM, "host buffer");
    }
    hipError_t e = hipMemcpyAsync(ctx->h_status, ctx->d_status, (TB_GSTAT_WORD + GS_WORDS) * sizeof(int), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess && want_loss) e = hipMemcpyAsync(host, L.lossbuf, 2 * (size_t)nh * sizeof(double), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { free(host); return tboa_fail(ctx, TBOA_EHIP, "status and loss copy: %s", hipGetErrorString(e)); }
    for (int slot = 0; slot <= (H_out ? 2 : 0); slot += 2)
        if (ctx->h_status[slot] != 0) {
            free(host);
            return tboa_fail(ctx, TBOA_ENOTSPD, "%s Hessian %d of the batch is not positive definite: pivot %d is not positive",
                             slot ? "out-channel" : "in-channel", ctx->h_status[slot + 1], ctx->h_status[slot] - 1);
        }
    if (L.fast_grid) {
        const int* gs = ctx->h_status + TB_GSTAT_WORD;
        float dev; memcpy(&dev, &gs[GS_MAXDEV], sizeof(float));
        ctx->counters[TBOA_CTR_GRID_SURVIVORS] += gs[GS_SURVIVORS];
        const double guard = d->grid_guard > 0.0 ? d->grid_guard : 0.25;
        if (gs[GS_TRIPPED] || dev > guard * GRID_TAU) { free(host); return RUN_AGAIN_EXACT; }
    }
    if (want_loss) {
        double q = 0.0, c = 0.0;
        for (int h = 0; h < nh; ++h) {
            q += host[h]; c += host[nh + h];
            if (loss_per_head) { loss_per_head[2 * h] = host[h]; loss_per_head[2 * h + 1] = host[nh + h]; }
        }
        if (loss) { loss[0] = q; loss[1] = c; }
        free(host);
        if (!(q == q) || !(c == c)) return tboa_fail(ctx, TBOA_ENAN, "quantize_layer: loss is not finite (non-finite input?)");
    }
    return 0;
}

// The workspace of a quantize_layer call, carved from `ar` (base == nullptr: only counted).
void plan_layer(Layer& L, bool H_out, bool R, Arena& ar) {
    const tboa_layer_desc* d = L.d;
    const int n = L.n, nh = L.nh, dh = L.dh;
    const int blk = d->block < dh ? d->block : dh;
    const size_t wn = (size_t)d->d_out * n, brows = (size_t)nh * blk;
    const size_t grows = (size_t)L.grid_chunk * (L.nhin > 1 ? (d->adaptive_grid ? blk : dh) : 1);
    const int fmax = n > dh ? n : dh;
    const int fb = (L.nhin > nh) ? L.nhin : nh;
    const int nblk_f = (fmax + TB_FACT_NB - 1) / TB_FACT_NB;
    L.W64 = ar.get<double>(wn); L.Wt = ar.get<double>(wn); L.Q64 = ar.get<double>(wn);
    L.s64 = ar.get<double>((size_t)d->d_out * L.ng); L.z64 = ar.get<double>((size_t)d->d_out * L.ng);
    L.Hi = ar.get<double>((size_t)L.nhin * L.nn); L.Hfac = ar.get<double>((size_t)L.nhin * L.nn); L.Uin = ar.get<double>((size_t)L.nhin * L.nn);
    L.Rd = R ? ar.get<double>((size_t)L.nhin * L.nn) : nullptr; L.P = R ? ar.get<double>((size_t)L.nhin * L.nn) : nullptr;
    L.Ho = H_out ? ar.get<double>((size_t)nh * dh * dh) : nullptr; L.Hofac = H_out ? ar.get<double>((size_t)nh * dh * dh) : nullptr;
    L.Uout = H_out ? ar.get<double>((size_t)nh * dh * dh) : nullptr;
    // the two factorisations (H_in: nhin matrices of order n; H_out: nh of order dh) share their temporaries
    const size_t t_in = (size_t)L.nhin * n * chol_tmp_pitch(n), t_out = H_out ? (size_t)nh * dh * chol_tmp_pitch(dh) : 0;
    L.ftmp = ar.get<double>(t_in > t_out ? t_in : t_out); L.fdinv = ar.get<double>((size_t)fb * nblk_f * TB_FACT_NB * TB_FACT_NB);
    L.Wb = ar.get<double>(brows * n); L.Wk = ar.get<double>(brows * n);
    L.Epan = ar.get<double>(brows * SWEEP_SP); L.Wsnap = ar.get<double>(brows * SWEEP_SP);
    L.E = H_out ? ar.get<double>(brows * n) : nullptr;
    L.S1 = (H_out && R) ? ar.get<double>(brows * n) : nullptr; L.S2 = (H_out && R) ? ar.get<double>(brows * n) : nullptr;
    L.T = H_out ? ar.get<double>((size_t)nh * dh * d->block) : nullptr;
    L.cand_s = ar.get<double>(grows * L.ncand); L.cand_z = ar.get<double>(grows * L.ncand); L.cost = ar.get<double>(grows * L.ncand);
    L.Delta = ar.get<double>(grows * L.ncand * L.gsz); L.G = ar.get<double>(grows * L.ncand * L.gsz);
    L.DeltaS = L.GS = L.costS = L.lim = nullptr; L.sel = nullptr; L.Hcat = nullptr;
    if (L.fast_grid) {
        L.DeltaS = ar.get<double>(grows * GRID_KS * n); L.GS = ar.get<double>(grows * GRID_KS * n);
        L.costS = ar.get<double>(grows * GRID_KS); L.lim = ar.get<double>(grows); L.sel = ar.get<int>(grows * 3);
        L.Hcat = ar.get<__hip_bfloat16>((size_t)L.nhin * n * (GRID_TERMS * (size_t)n + GRID_PAD));
    }
    L.Wbar = ar.get<double>(wn); L.Abar = ar.get<double>(wn); L.Z = ar.get<double>(wn);
    L.WR = R ? ar.get<double>(wn) : nullptr;
    L.Cm = H_out ? ar.get<double>((size_t)nh * dh * dh) : nullptr; L.Fm = H_out ? ar.get<double>((size_t)nh * dh * dh) : nullptr;
    L.dvec = ar.get<double>(2 * (size_t)d->d_out); L.lossbuf = ar.get<double>(2 * (size_t)nh);
    L.Cg = L.Fg = nullptr;
    if (d->group && d->cd_iters > 0) {
        const size_t ng = (size_t)L.ng;
        L.Cg = ar.get<double>(H_out ? (size_t)nh * ng * ng * dh * dh : (size_t)d->d_out * ng * ng);
        L.Fg = ar.get<double>(H_out ? (size_t)nh * ng * dh * dh : (size_t)d->d_out * ng);
    }
}

int check_layer_desc(tboa_ctx* ctx, const tboa_layer_desc* d) {
    if (!d) return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: null descriptor");
    if (d->d_out <= 0 || d->d_in <= 0 || d->n_heads <= 0 || d->d_out % d->n_heads != 0)
        return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: d_out=%d must be a positive multiple of n_heads=%d", d->d_out, d->n_heads);
    if (!(d->bits == 2 || d->bits == 3 || d->bits == 4 || d->bits == 8)) return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: bits=%d not in {2,3,4,8}", d->bits);
    if (d->block <= 0) return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: block must be positive");
    if (d->group < 0 || (d->group > 0 && d->d_in % d->group != 0)) return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: group=%d must divide d_in=%d", d->group, d->d_in);
    if (d->group > 0 && !(d->group % 64 == 0 || 64 % d->group == 0)) return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: group=%d must divide or be a multiple of 64", d->group);
    if (d->w_dtype != TBOA_F32 && d->w_dtype != TBOA_BF16) return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: w_dtype");
    if (d->grid_points <= 0 || !(d->max_shrink > 0.0) || d->max_shrink > 1.0 || d->damp < 0.0 || d->cd_iters < 0 || !(d->grid_guard == d->grid_guard))
        return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: grid_points/max_shrink/damp/cd_iters/grid_guard out of range");
    return 0;
}

// the quantities of a layer that follow from its descriptor alone
void init_layer(Layer& L, tboa_ctx* ctx, const tboa_layer_desc* d) {
    L.ctx = ctx; L.d = d;
    L.n = d->d_in; L.nh = d->n_heads; L.dh = d->d_out / d->n_heads;
    L.ng = d->group ? d->d_in / d->group : 1; L.gsz = d->group ? d->group : d->d_in;
    L.nhin = d->hin_per_head ? d->n_heads : 1;
    L.ncand = (int)ceil(d->max_shrink * (double)d->grid_points);
    if (L.ncand < 1) L.ncand = 1;
    L.maxq = (double)((1 << d->bits) - 1);
    L.nn = (long long)L.n * L.n;
    const int blk = d->block < L.dh ? d->block : L.dh;
    // grid-search pass size: keep Delta and G near 2 GiB each
    const double cap = 2147483648.0;
    const double per_row = (double)L.ncand * L.gsz * 8.0;
    const int max_rows_block = d->adaptive_grid ? blk : L.dh;
    if (L.nhin > 1) { int c = (int)(cap / (per_row * max_rows_block)); L.grid_chunk = c < 1 ? 1 : (c > L.nh ? L.nh : c); }
    else { int c = (int)(cap / per_row); const int tot = L.nh * max_rows_block; L.grid_chunk = c < 1 ? 1 : (c > tot ? tot : c); }
    // per-row grids of wide layers: two-phase search (a negative grid_guard asks for exact costs throughout); its GEMM
    // operands in 16 x 32 blocks when the width allows
    L.fast_grid = (!d->group && L.n % 8 == 0 && L.n >= 256 && !(d->grid_guard < 0.0)) ? 1 : 0;
    L.grid_blocked = (L.fast_grid && L.n % 32 == 0) ? 1 : 0;
    L.gstat = ctx ? ctx->d_status + TB_GSTAT_WORD : nullptr;
}

}  // namespace

extern "C" size_t tboa_quantize_workspace_bytes(const tboa_layer_desc* d, int with_H_out, int with_R) {
    if (check_layer_desc(nullptr, d) != 0) return 0;
    Layer L{};
    init_layer(L, nullptr, d);
    Arena ar(nullptr);
    plan_layer(L, with_H_out != 0, with_R != 0, ar);
    return ar.off;
}

extern "C" int tboa_quantize_layer(tboa_ctx* ctx, const tboa_layer_desc* d, const void* W, const float* H_in, const float* H_out,
                                   const float* R, uint8_t* codes, float* scales, float* zeros, float* W_deq, double* loss,
                                   double* loss_per_head) {
    if (!ctx) return TBOA_EINVAL;
    if (!d || !W || !H_in || !codes || !scales || !zeros || !W_deq) return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: null argument");
    TB_TRY(check_layer_desc(ctx, d));
    if (d->hin_per_head && d->n_heads > 1 && !H_out) return tboa_fail(ctx, TBOA_EINVAL, "quantize_layer: per-head H_in needs H_out");

    Layer L{};
    init_layer(L, ctx, d);
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        plan_layer(L, H_out != nullptr, R != nullptr, ar);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    int rc = run_layer(L, W, H_in, H_out, R, codes, scales, zeros, W_deq, loss, loss_per_head);
    if (rc == RUN_AGAIN_EXACT) {
        // the guard of the two-phase grid search: exact costs for every candidate, same workspace
        ++ctx->counters[TBOA_CTR_GRID_FALLBACKS];
        L.fast_grid = 0;
        rc = run_layer(L, W, H_in, H_out, R, codes, scales, zeros, W_deq, loss, loss_per_head);
    }
    return rc;
}
