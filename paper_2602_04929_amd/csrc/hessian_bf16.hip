// Table 1 Hessians for bf16 inputs, on the bf16 matrix cores, and the public entry points of the Hessian build.
//
// Every contraction is brought into the one shape the bf16 GEMM kernel has (both operands contiguous along the
// contraction axis):
//   H_in = X X^T            A = B = X^T [d, T]                     (split over T, partial sums reduced in fp64)
//   R    = alpha dX X^T     A = dX^T as an exact hi + lo bf16 pair, B = X^T
//   Q, K projections        A = X rows [tokens, d], B = W [out, d]  -> fp32, then split into (hi, lo) pairs of 16-bit values so that
//   scores Q_h K_h^T        runs as one product over [hi | lo | hi] . [hi | hi | lo] (peaked softmaxes need the accuracy, and the
//                           difference A - A~ of two softmaxes more still: where the fused scores + softmax kernel runs the pairs
//                           are IEEE half values of the projections times a power of two, 22 significant bits; the GEMM path
//                           takes bf16 pairs, 16 bits)
//   Y_h^T = X_s^T A_h^T     A = X_s^T [d, L], B = A_h [L, L] (lower triangular: the k-loop stops at the diagonal tile)
//   H_in^V += Y^T (Y^T)^T   A = B = Y^T [d, rep*G*L] for G sequences at a time, lower tiles only
//   R_v += alpha dY^T (Y^T)^T with dY^T = [X_s^T | X~_s^T] . [A | -A~]^T taken from ONE fp32 accumulator
// The L x L probabilities are materialised per sequence (bf16, a few hundred MB for all heads): with 288 GB of HBM
// and a value dimension of d_model the traffic is negligible next to the flops.
// H_out of W_Q / W_K / W_V are tiny Gram matrices, computed in fp64 from H_in and the weights
// (K_h^T K_h = W_K,h H_in W_K,h^T exactly, there being no positional rotation in the block).
#include "internal.h"
#include <math.h>
#include <stdlib.h>

int gemm_bf16_nt(tboa_ctx* ctx, const GemmBf16& g);

namespace {

typedef __hip_bfloat16 bf16;

// Operands of the W_V and W_O Hessian chains (probabilities, transposed activations, A X) are 16-bit values of one of two
// kinds, chosen per call: IEEE half (11 significant bits; the default) or bf16 (8 bits; taken when an activation exceeds the
// range of half).  Buffers are typed bf16 either way; these helpers produce and read the bits.
__device__ __forceinline__ bf16 enc16(float v, int f16) {
    if (f16) { const _Float16 h = (_Float16)v; return __builtin_bit_cast(bf16, h); }
    return __float2bfloat16(v);
}
__device__ __forceinline__ float dec16(bf16 b, int f16) {
    if (f16) return (float)__builtin_bit_cast(_Float16, b);
    return __bfloat162float(b);
}

// out[c, r] = in[r, c] (optionally also the hi/lo split of in - in2), 64 x 64 tiles through LDS; blocked: the
// outputs are kept in 16 x 32 blocks; f16: the outputs are IEEE half (the inputs are always bf16)
__global__ __launch_bounds__(256) void transpose_kernel(const bf16* __restrict__ in, const bf16* __restrict__ in2, long long ld_in,
                                                        int rows, int cols, bf16* __restrict__ out, bf16* __restrict__ out_hi,
                                                        bf16* __restrict__ out_lo, long long ld_out, int blocked, int vec, int f16) {
    __shared__ float t0[64][65];
    __shared__ float t1[64][65];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    if (vec && r0 + 64 <= rows && c0 + 64 <= cols) {
        // whole tile: 16-byte loads of 8 consecutive input columns, 16-byte stores of 8 consecutive input rows (one chunk of a
        // 16 x 32 block, or of an output row)
        for (int i = threadIdx.x; i < 512; i += 256) {
            const int r = i >> 3, c = (i & 7) * 8;
            union { uint4 u; bf16 b[8]; } a, b2;
            a.u = *(const uint4*)(in + (long long)(r0 + r) * ld_in + c0 + c);
            if (in2) b2.u = *(const uint4*)(in2 + (long long)(r0 + r) * ld_in + c0 + c);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float v = __bfloat162float(a.b[j]);
                t0[r][c + j] = v; t1[r][c + j] = in2 ? v - __bfloat162float(b2.b[j]) : v;
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < 512; i += 256) {
            const int c = i >> 3, r = (i & 7) * 8;
            const long long o = blocked ? tboa_blocked_offset(c0 + c, r0 + r, ld_out >> 5) : (long long)(c0 + c) * ld_out + r0 + r;
            union { uint4 u; bf16 b[8]; } x, hi, lo;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                x.b[j] = enc16(t0[r + j][c], f16);
                const float dlt = t1[r + j][c];
                hi.b[j] = enc16(dlt, f16);
                lo.b[j] = enc16(dlt - dec16(hi.b[j], f16), f16);
            }
            if (out) *(uint4*)(out + o) = x.u;
            if (out_hi) { *(uint4*)(out_hi + o) = hi.u; if (out_lo) *(uint4*)(out_lo + o) = lo.u; }
        }
        return;
    }
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int r = i >> 6, c = i & 63;
        float v = 0.f, w = 0.f;
        if (r0 + r < rows && c0 + c < cols) {
            v = __bfloat162float(in[(long long)(r0 + r) * ld_in + c0 + c]);
            if (in2) w = __bfloat162float(in2[(long long)(r0 + r) * ld_in + c0 + c]);
        }
        t0[r][c] = v; t1[r][c] = v - w;     // the difference of two bf16 values is exact in fp32
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int c = i >> 6, r = i & 63;
        if (r0 + r < rows && c0 + c < cols) {
            const long long o = blocked ? tboa_blocked_offset(c0 + c, r0 + r, ld_out >> 5) : (long long)(c0 + c) * ld_out + r0 + r;
            if (out) out[o] = enc16(t0[r][c], f16);
            if (out_hi) {
                const float dlt = t1[r][c];
                const bf16 hi = enc16(dlt, f16);
                out_hi[o] = hi;
                if (out_lo) out_lo[o] = enc16(dlt - dec16(hi, f16), f16);
            }
        }
    }
}

// fp32 [rows, H*dh] -> bf16 [rows, H, 3*dh]: (hi, lo, hi) for the left operand, (hi, hi, lo) for the right one;
// scale (or NULL): one factor per column of `in`, applied first (projections through integer-form weights).
// L > 0: the rows are whole sequences of L tokens and the result is one [L, 3*dh] matrix per (sequence, head), each in the
// 16 x 32 blocks the bf16 GEMM reads (L a multiple of 16, 3*dh of 32): element (t, c) of sequence s, head h at
// ((s H + h) L 3dh) + tboa_blocked_offset(t, c, 3dh / 32).
// amax (blocked result only, else NULL): one word per sequence as amax_seq_kernel leaves it; the pairs of that sequence are
// then IEEE half values of the input times 2^tboa_half_exp(word) instead of bf16 (see QkScale).
__device__ __forceinline__ long long split3_offset(long long row, int h, int c, int H, int dh, int L) {
    if (L > 0) return ((row / L) * H + h) * (long long)L * 3 * dh + tboa_blocked_offset(row % L, c, (3 * dh) >> 5);
    return (row * H + h) * 3 * dh + c;
}

__global__ void split3_kernel(const float* __restrict__ in, const float* __restrict__ scale, bf16* __restrict__ out, long long rows, int hd,
                              int dh, int right, int L, const int* __restrict__ amax) {
    const int H = hd / dh;
    if (L > 0 && dh % 32 == 0 && rows % 16 == 0 && rows / 16 * (hd / 32) < 2147483647LL) {
        // blocked result: a wavefront takes a 16 x 32 piece of `in` in two loads of eight whole rows of 128 bytes (lane: row
        // lane / 8 and that row + 8, four columns from 4 (lane % 8)) and writes the three 1 KB blocks it becomes, each as two
        // contiguous halves of 512 bytes.  Everything but the lane's place inside the block is uniform over the wavefront
        // (32-bit scalar arithmetic).
        typedef float f4 __attribute__((ext_vector_type(4)));
        const int lane = threadIdx.x & 63, ri = lane >> 3, c4 = (lane & 7) * 4;
        const unsigned cbs = hd / 32, nblk = (unsigned)(rows / 16) * cbs, nw = gridDim.x * (blockDim.x >> 6);
        const unsigned in_lane = ri * hd + c4, kb = (3 * dh) >> 5;
        // rows ri and ri + 8 of the block: the 16-byte piece c4 / 8 is permuted with (row / 4) % 4
        const unsigned out_a = ri * 32 + (((c4 >> 3) ^ (ri >> 2)) << 3) + (c4 & 7), out_b = (ri + 8) * 32 + (((c4 >> 3) ^ ((ri + 8) >> 2)) << 3) + (c4 & 7);
        for (unsigned b = __builtin_amdgcn_readfirstlane(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)); b < nblk; b += nw) {
            const unsigned rb = b / cbs, c0 = (b % cbs) * 32, h = c0 / dh, e0 = c0 % dh;
            const unsigned row0 = rb * 16, sq = row0 / (unsigned)L, t0 = row0 % (unsigned)L;
            const float* src = in + (long long)row0 * hd + c0 + in_lane;
            f4 va = __builtin_nontemporal_load((const f4*)src), vb = __builtin_nontemporal_load((const f4*)(src + 8LL * hd));
            if (scale) { const f4 sc = *(const f4*)(scale + c0 + c4); va = va * sc; vb = vb * sc; }
            union { bf16 b[4]; uint2 u; } ha, la, hb, lb;
            const int word = amax ? amax[sq] : -1;
            if (word >= 0) {
                const float up = ldexpf(1.f, tboa_half_exp(word));
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float a = va[k] * up, b2 = vb[k] * up;
                    ha.b[k] = enc16(a, 1); la.b[k] = enc16(a - dec16(ha.b[k], 1), 1);
                    hb.b[k] = enc16(b2, 1); lb.b[k] = enc16(b2 - dec16(hb.b[k], 1), 1);
                }
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    ha.b[k] = __float2bfloat16(va[k]); la.b[k] = __float2bfloat16(va[k] - __bfloat162float(ha.b[k]));
                    hb.b[k] = __float2bfloat16(vb[k]); lb.b[k] = __float2bfloat16(vb[k] - __bfloat162float(hb.b[k]));
                }
            }
            // block (t0 / 16, (seg dh + e0) / 32) of the [L, 3 dh] matrix of (sequence sq, head h)
            bf16* o = out + ((long long)sq * H + h) * L * 3 * dh + ((long long)(t0 >> 4) * kb + (e0 >> 5)) * 512;
            const long long seg = (long long)(dh >> 5) * 512;
            *(uint2*)(o + out_a) = ha.u; *(uint2*)(o + out_b) = hb.u;
            *(uint2*)(o + seg + out_a) = right ? ha.u : la.u; *(uint2*)(o + seg + out_b) = right ? hb.u : lb.u;
            *(uint2*)(o + 2 * seg + out_a) = right ? la.u : ha.u; *(uint2*)(o + 2 * seg + out_b) = right ? lb.u : hb.u;
        }
        return;
    }
    if (hd % 4 == 0 && dh % 4 == 0) {     // four consecutive columns per thread: 16-byte streaming loads, 8-byte stores
        typedef float f4 __attribute__((ext_vector_type(4)));
        const long long tot4 = rows * hd / 4;
        const int hd4 = hd / 4;
        for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < tot4; i += (long long)gridDim.x * blockDim.x) {
            const long long row = i / hd4; const int c = (int)(i % hd4) * 4, h = c / dh, e = c % dh;
            f4 v = __builtin_nontemporal_load((const f4*)(in + 4 * i));
            if (scale) { const f4 sc = *(const f4*)(scale + c); v = v * sc; }
            union { bf16 b[4]; uint2 u; } hi, lo;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                hi.b[j] = __float2bfloat16(v[j]);
                lo.b[j] = __float2bfloat16(v[j] - __bfloat162float(hi.b[j]));
            }
            *(uint2*)(out + split3_offset(row, h, e, H, dh, L)) = hi.u;
            *(uint2*)(out + split3_offset(row, h, dh + e, H, dh, L)) = right ? hi.u : lo.u;
            *(uint2*)(out + split3_offset(row, h, 2 * dh + e, H, dh, L)) = right ? lo.u : hi.u;
        }
        return;
    }
    const long long tot = rows * hd;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < tot; i += (long long)gridDim.x * blockDim.x) {
        const long long row = i / hd; const int c = (int)(i % hd), h = c / dh, e = c % dh;
        const float v = scale ? in[i] * scale[c] : in[i];
        const bf16 hi = __float2bfloat16(v);
        const bf16 lo = __float2bfloat16(v - __bfloat162float(hi));
        out[split3_offset(row, h, e, H, dh, L)] = hi;
        out[split3_offset(row, h, dh + e, H, dh, L)] = right ? hi : lo;
        out[split3_offset(row, h, 2 * dh + e, H, dh, L)] = right ? lo : hi;
    }
}

// out[s] = bits of the largest |in[r, c] scale[c]| over the rows of sequence s (blockIdx.y; L rows of hd columns each), by
// atomicMax on the integer: a word that starts negative ends as those bits.  A NaN counts as infinity.
__global__ __launch_bounds__(256) void amax_seq_kernel(const float* __restrict__ in, const float* __restrict__ scale, int L, int hd,
                                                       int* __restrict__ out) {
    const float* src = in + (long long)blockIdx.y * L * hd;
    const long long n = (long long)L * hd;
    float m = 0.f;
    auto take = [&](float v) { v = fabsf(v); m = (v > m || !(v == v)) ? (v == v ? v : INFINITY) : m; };
    const long long tid = blockIdx.x * (long long)blockDim.x + threadIdx.x, nth = (long long)gridDim.x * blockDim.x;
    if (hd % 4 == 0 && (((uintptr_t)in | (uintptr_t)scale) & 15) == 0) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        for (long long i = tid; i < n / 4; i += nth) {
            f4 v = *((const f4*)src + i);
            if (scale) v = v * *(const f4*)(scale + (4 * i) % hd);
            take(v.x); take(v.y); take(v.z); take(v.w);
        }
    } else
        for (long long i = tid; i < n; i += nth) take(scale ? src[i] * scale[i % hd] : src[i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    __shared__ float red[4];      // one atomic per workgroup: they all land on the sequence's one word
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) atomicMax(out + blockIdx.y, __float_as_int(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]))));
}

// fp32 [n] -> three bf16 terms whose sum is the value to 24 bits
__global__ void split_three_kernel(const float* __restrict__ in, bf16* __restrict__ hi, bf16* __restrict__ mid, bf16* __restrict__ lo, long long n) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
        const float v = in[i];
        const bf16 h = __float2bfloat16(v);
        const float r = v - __bfloat162float(h);
        const bf16 m = __float2bfloat16(r);
        hi[i] = h; mid[i] = m; lo[i] = __float2bfloat16(r - __bfloat162float(m));
    }
}

// fp32 [n] -> exact-to-16-bits pair of bf16
__global__ void split_hilo_kernel(const float* __restrict__ in, bf16* __restrict__ hi, bf16* __restrict__ lo, long long n) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
        const float v = in[i];
        const bf16 h = __float2bfloat16(v);
        hi[i] = h; lo[i] = __float2bfloat16(v - __bfloat162float(h));
    }
}

// Integer form of a dequantized weight.  A row of W_deq = s (codes - z) holds integer multiples of its scale, and small
// integers are exact in bf16: X W_deq^T = (X K^T) diag(step) with K = W_deq / step needs ONE bf16 GEMM with exact operands,
// where the general (hi, lo) split of an fp32 weight needs two.  One workgroup per row takes the greatest common divisor
// (Euclid's algorithm on floats, remainders below 1e-3 of the divisor counting as zero) of the distances of the entries
// from the row minimum, checks that every entry is a multiple k of it with |k| <= 256 (up to fp32 rounding of the
// entries: with |k| <= 256 a true remainder is at least 1/256 of the divisor), and refines the step as the least-squares
// fit sum(w k) / sum(k k).  A row that is not of this form (weights that are not a dequantized uniform grid, group-wise
// scales, a row whose used levels all sit a common factor apart from zero) raises *fail, and the caller keeps the
// (hi, lo) path for the whole matrix.
__device__ __forceinline__ float float_gcd(float a, float b) {
    if (a == 0.f) return b;
    if (b == 0.f) return a;
    if (a < b) { const float t = a; a = b; b = t; }
    for (int it = 0; it < 32; ++it) {
        const float r = fabsf(a - b * rintf(a / b));
        if (r <= 1e-3f * b) return b;
        a = b; b = r;
    }
    return b;
}

__global__ __launch_bounds__(256) void int_form_kernel(const float* __restrict__ W, int n, bf16* __restrict__ K, float* __restrict__ step,
                                                       int* __restrict__ fail) {
    __shared__ float red[4]; __shared__ double redd[8];
    const float* w = W + (long long)blockIdx.x * n;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    float m = INFINITY;
    for (int c = threadIdx.x; c < n; c += 256) m = fminf(m, w[c]);
    for (int o = 32; o > 0; o >>= 1) m = fminf(m, __shfl_xor(m, o, 64));
    if (lane == 0) red[wv] = m;
    __syncthreads();
    m = fminf(fminf(red[0], red[1]), fminf(red[2], red[3]));
    __syncthreads();
    float d = fabsf(m);          // the minimum itself is a multiple of the step too
    for (int c = threadIdx.x; c < n; c += 256) d = float_gcd(d, w[c] - m);
    for (int o = 32; o > 0; o >>= 1) d = float_gcd(d, __shfl_xor(d, o, 64));
    if (lane == 0) red[wv] = d;
    __syncthreads();
    d = float_gcd(float_gcd(red[0], red[1]), float_gcd(red[2], red[3]));
    if (!(d > 0.f)) d = 1.f;     // an all-zero row
    bool ok = true;
    double swk = 0.0, skk = 0.0;
    for (int c = threadIdx.x; c < n; c += 256) {
        const float k = w[c] / d, kr = rintf(k);
        if (!(fabsf(k - kr) <= 1e-3f) || fabsf(kr) > 256.f) ok = false;
        swk += (double)w[c] * kr; skk += (double)kr * kr;
    }
    for (int o = 32; o > 0; o >>= 1) { swk += __shfl_xor(swk, o, 64); skk += __shfl_xor(skk, o, 64); }
    if (lane == 0) { redd[wv] = swk; redd[4 + wv] = skk; }
    const int all_ok = __syncthreads_and(ok);
    swk = redd[0] + redd[1] + redd[2] + redd[3]; skk = redd[4] + redd[5] + redd[6] + redd[7];
    const float st = skk > 0.0 ? (float)(swk / skk) : d;
    for (int c = threadIdx.x; c < n; c += 256) K[(long long)blockIdx.x * n + c] = __float2bfloat16(rintf(w[c] / d));
    if (threadIdx.x == 0) { step[blockIdx.x] = st; if (!all_ok || !(st > 0.f)) atomicOr(fail, 1); }
}

// V^T fp32 [rows, G*L] (times row_scale, if given) -> per-sequence segments of length L: (hi, hi, lo) of V^T in segments
// 0, 1, 2 and, when the full-precision V~^T is given, (hi, hi, lo) of V~^T in segments 3, 4, 5
__global__ void vt_segments_kernel(const float* __restrict__ in, const float* __restrict__ row_scale, const float* __restrict__ in_fp,
                                   bf16* __restrict__ out, int rows, int G, int L, int nseg, long long ld, int f16) {
    const long long tot = (long long)rows * G * L;
    if (L % 4 == 0 && ld % 4 == 0 && ((uintptr_t)out & 7) == 0) {     // four consecutive tokens per thread: 16-byte streaming loads, 8-byte stores
        typedef float f4 __attribute__((ext_vector_type(4)));
        for (long long i4 = blockIdx.x * (long long)blockDim.x + threadIdx.x; i4 < tot / 4; i4 += (long long)gridDim.x * blockDim.x) {
            const long long i = 4 * i4, row = i / ((long long)G * L); const int s = (int)((i / L) % G), t = (int)(i % L);
            f4 v = __builtin_nontemporal_load((const f4*)(in + i));
            if (row_scale) v = v * row_scale[row];
            f4 w = {0.f, 0.f, 0.f, 0.f};
            if (in_fp) w = __builtin_nontemporal_load((const f4*)(in_fp + i));
            union { bf16 b[4]; uint2 u; } h, l, wh, wl;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                h.b[j] = enc16(v[j], f16); l.b[j] = enc16(v[j] - dec16(h.b[j], f16), f16);
                wh.b[j] = enc16(w[j], f16); wl.b[j] = enc16(w[j] - dec16(wh.b[j], f16), f16);
            }
            bf16* o = out + row * ld + ((long long)s * nseg) * L + t;
            *(uint2*)o = h.u; *(uint2*)(o + L) = h.u; *(uint2*)(o + 2 * L) = l.u;
            if (in_fp) { *(uint2*)(o + 3 * L) = wh.u; *(uint2*)(o + 4 * L) = wh.u; *(uint2*)(o + 5 * L) = wl.u; }
        }
        return;
    }
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < tot; i += (long long)gridDim.x * blockDim.x) {
        const long long row = i / ((long long)G * L); const int s = (int)((i / L) % G), t = (int)(i % L);
        const float v = row_scale ? in[i] * row_scale[row] : in[i];
        const bf16 h = enc16(v, f16);
        bf16* o = out + row * ld + ((long long)s * nseg) * L + t;
        o[0] = h; o[L] = h; o[2 * L] = enc16(v - dec16(h, f16), f16);
        if (in_fp) { const float w = in_fp[i]; const bf16 wh = enc16(w, f16); o[3 * L] = wh; o[4 * L] = wh; o[5 * L] = enc16(w - dec16(wh, f16), f16); }
    }
}

// P[t, k] = A[t, k] (and once more at column hi2col + k, and its low part A - P[t, k] at locol + k, when those are not
// negative), A = softmax over the first t+1 (causal) or L entries of the score row; with a
// second score matrix S2 also P[t, dcol + k] = A[t, k] - A2[t, k], the difference taken in fp32 before rounding, or
// (pair2) A2 itself as (hi, lo, hi) in the three segments of L columns from dcol.
// Zero up to the next multiple of 256 (the k-loop of the consumer stops there).  One wavefront per row, y = head.
__global__ __launch_bounds__(256) void softmax_bf16_kernel(const float* __restrict__ S, const float* __restrict__ S2, int L, int causal,
                                                           bf16* __restrict__ P, long long ldp, long long head_stride, int hi2col, int locol, int dcol, int f16,
                                                           int pair2) {
    const int lane = threadIdx.x & 63, t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= L) return;
    const long long so = ((long long)blockIdx.y * L + t) * L;
    const float* s = S + so; const float* s2 = S2 ? S2 + so : nullptr;
    bf16* p = P + blockIdx.y * head_stride + (long long)t * ldp;
    const int kend = causal ? t + 1 : L;
    int kz = ((kend + 255) / 256) * 256; if (kz > L) kz = L;
    float m = -INFINITY, m2 = -INFINITY;
    for (int k = lane; k < kend; k += 64) { m = fmaxf(m, s[k]); if (s2) m2 = fmaxf(m2, s2[k]); }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { m = fmaxf(m, __shfl_xor(m, o, 64)); m2 = fmaxf(m2, __shfl_xor(m2, o, 64)); }
    float sum = 0.f, sum2 = 0.f;
    for (int k = lane; k < kend; k += 64) { sum += __expf(s[k] - m); if (s2) sum2 += __expf(s2[k] - m2); }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { sum += __shfl_xor(sum, o, 64); sum2 += __shfl_xor(sum2, o, 64); }
    const float inv = 1.f / sum, inv2 = s2 ? 1.f / sum2 : 0.f;
    for (int k = lane; k < kz; k += 64) {
        const float a = k < kend ? __expf(s[k] - m) * inv : 0.f;
        const bf16 v = enc16(a, f16);
        p[k] = v;
        if (hi2col >= 0) p[hi2col + k] = v;
        if (locol >= 0) p[locol + k] = enc16(a - dec16(v, f16), f16);
        if (s2) {
            const float a2 = k < kend ? __expf(s2[k] - m2) * inv2 : 0.f;
            if (pair2) { const bf16 v2 = enc16(a2, f16); p[dcol + k] = v2; p[dcol + L + k] = enc16(a2 - dec16(v2, f16), f16); p[dcol + 2 * L + k] = v2; }
            else p[dcol + k] = enc16(a - a2, f16);
        }
    }
}

// Same result layout as softmax_bf16_kernel for rows of at most 256 * NCH scores (L a multiple of 4): the row is read
// once with 16-byte loads and kept in registers (lane l holds scores 256 c + 4 l .. + 3 of chunk c), each exponential
// is taken once, and the probabilities leave as 8-byte stores.
template <int NCH>
__global__ __launch_bounds__(256) void softmax_bf16_regs_kernel(const float* __restrict__ S, const float* __restrict__ S2, int L, int causal,
                                                                bf16* __restrict__ P, long long ldp, long long head_stride, int hi2col, int locol, int dcol,
                                                                int blocked, int f16, int pair2) {
    const int lane = threadIdx.x & 63, t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= L) return;
    // heads from the last to the first: the score product wrote them in ascending order, so the last ones are the part of the
    // scores the memory-side cache still holds (measured: 175 -> 169 us on 32 heads x 2048^2)
    const int hy = gridDim.y - 1 - blockIdx.y;
    const long long so = ((long long)hy * L + t) * L;
    const float* s = S + so; const float* s2 = S2 ? S2 + so : nullptr;
    bf16* p = P + hy * head_stride + (blocked ? 0 : (long long)t * ldp);
    const int kend = causal ? t + 1 : L;
    int kz = ((kend + 255) / 256) * 256; if (kz > L) kz = L;
    float v[NCH][4], w[NCH][4];
    float m = -INFINITY, m2 = -INFINITY;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int k = c * 256 + lane * 4;
        float4 a = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY), b = a;
        if (k < kz) {     // the scores are read this once: streaming loads leave the L2 to the probabilities being written
            typedef float f4 __attribute__((ext_vector_type(4)));
            const f4 ta = __builtin_nontemporal_load((const f4*)(s + k)); a = make_float4(ta.x, ta.y, ta.z, ta.w);
            if (s2) { const f4 tb = __builtin_nontemporal_load((const f4*)(s2 + k)); b = make_float4(tb.x, tb.y, tb.z, tb.w); }
        }
        v[c][0] = a.x; v[c][1] = a.y; v[c][2] = a.z; v[c][3] = a.w;
        w[c][0] = b.x; w[c][1] = b.y; w[c][2] = b.z; w[c][3] = b.w;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (k + i >= kend) { v[c][i] = -INFINITY; w[c][i] = -INFINITY; }
            m = fmaxf(m, v[c][i]); m2 = fmaxf(m2, w[c][i]);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { m = fmaxf(m, __shfl_xor(m, o, 64)); m2 = fmaxf(m2, __shfl_xor(m2, o, 64)); }
    float sum = 0.f, sum2 = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[c][i] = __expf(v[c][i] - m); sum += v[c][i];
            if (s2) { w[c][i] = __expf(w[c][i] - m2); sum2 += w[c][i]; }
        }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { sum += __shfl_xor(sum, o, 64); sum2 += __shfl_xor(sum2, o, 64); }
    const float inv = 1.f / sum, inv2 = s2 ? 1.f / sum2 : 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int k = c * 256 + lane * 4;
        if (k >= kz) continue;
        union { bf16 h[4]; uint2 u; } pa, pl, pd, pe;       // pd: A - A2, or (pair2) the high part of A2 with its low part in pe
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = v[c][i] * inv, a2 = s2 ? w[c][i] * inv2 : 0.f;
            pa.h[i] = enc16(a, f16);
            pl.h[i] = enc16(a - dec16(pa.h[i], f16), f16);
            pd.h[i] = enc16(pair2 ? a2 : (s2 ? a - a2 : 0.f), f16);
            pe.h[i] = enc16(a2 - dec16(pd.h[i], f16), f16);
        }
        if (blocked) {     // the head's [L, ldp] matrix in 16 x 32 blocks: 4 consecutive columns stay together
            *(uint2*)(p + tboa_blocked_offset(t, k, ldp >> 5)) = pa.u;
            if (hi2col >= 0) *(uint2*)(p + tboa_blocked_offset(t, (long long)hi2col + k, ldp >> 5)) = pa.u;
            if (locol >= 0) *(uint2*)(p + tboa_blocked_offset(t, (long long)locol + k, ldp >> 5)) = pl.u;
            if (s2) *(uint2*)(p + tboa_blocked_offset(t, dcol + k, ldp >> 5)) = pd.u;
            if (s2 && pair2) {
                *(uint2*)(p + tboa_blocked_offset(t, (long long)dcol + L + k, ldp >> 5)) = pe.u;
                *(uint2*)(p + tboa_blocked_offset(t, (long long)dcol + 2 * L + k, ldp >> 5)) = pd.u;
            }
        } else {
            *(uint2*)(p + k) = pa.u;
            if (hi2col >= 0) *(uint2*)(p + hi2col + k) = pa.u;
            if (locol >= 0) *(uint2*)(p + locol + k) = pl.u;
            if (s2) *(uint2*)(p + dcol + k) = pd.u;
            if (s2 && pair2) { *(uint2*)(p + dcol + L + k) = pe.u; *(uint2*)(p + dcol + 2 * L + k) = pd.u; }
        }
    }
}

// Transposed probabilities, for the form of the W_V Hessian that sums over the query heads of a KV group before the wide
// products:  Pt[g][i][r L + t] = A_h[t, i] and dPt[g][i][r L + t] = A_h[t, i] - A~_h[t, i] with h = g rep + r, each as an
// exact-to-twice-the-mantissa (hi, lo) pair of 16-bit values; every [L, rep L (+ pad)] matrix of a group is kept in
// 16 x 32 blocks.  One workgroup per (64 rows t, head): the statistics of its rows first (one pass, running maximum and
// rescaled sum; a wavefront takes 16 rows), then the 64 x 64 pieces of the scores are read again, turned into
// probabilities and written transposed through LDS.  The rows i up to the end of the 256-tile that holds t are written,
// zeros beyond the diagonal: a product that starts its contraction at the 256-tile of its rows and columns
// (TBOA_GEMM_KLO) reads nothing else.  Causal scores with valid lower 256-tiles, L a multiple of 256.

__global__ __launch_bounds__(256) void softmax_t_kernel(const float* __restrict__ S, const float* __restrict__ S2, int L, int rep,
                                                        PtOut out, long long ldp, long long group_stride, int f16) {
    __shared__ float st[4][64];                                      // max, 1 / sum of the two score matrices, per row
    __shared__ __attribute__((aligned(16))) bf16 tp[4][64][72];      // [part][i][t]: hi, lo of A, hi, lo of A - A~; rows of 144 bytes
    const int h = gridDim.y - 1 - blockIdx.y, t0 = blockIdx.x * 64;      // heads from the last: their scores were written last
    const int g = h / rep, r = h % rep;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float* s = S + (long long)h * L * L;
    const float* s2 = S2 ? S2 + (long long)h * L * L : nullptr;
    typedef float f4 __attribute__((ext_vector_type(4)));
    for (int rr = 0; rr < 16; ++rr) {
        const int tl = wave * 16 + rr, t = t0 + tl;
        const float* row = s + (long long)t * L; const float* row2 = s2 ? s2 + (long long)t * L : nullptr;
        // one pass, four consecutive scores per lane and step: running maximum and rescaled sum per lane, merged at the end
        float m = -INFINITY, sum = 0.f, m2 = -INFINITY, sum2 = 0.f;
        for (int k = 4 * lane; k <= t; k += 256) {
            const f4 v = *(const f4*)(row + k);
            f4 w = {0.f, 0.f, 0.f, 0.f};
            if (row2) w = *(const f4*)(row2 + k);
            float vm = -INFINITY, wm = -INFINITY;
#pragma unroll
            for (int e = 0; e < 4; ++e) if (k + e <= t) { vm = fmaxf(vm, v[e]); wm = fmaxf(wm, w[e]); }
            if (vm > m) { sum *= __expf(m - vm); m = vm; }
            if (row2 && wm > m2) { sum2 *= __expf(m2 - wm); m2 = wm; }
#pragma unroll
            for (int e = 0; e < 4; ++e) if (k + e <= t) { sum += __expf(v[e] - m); if (row2) sum2 += __expf(w[e] - m2); }
        }
        float M = m, M2 = m2;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) { M = fmaxf(M, __shfl_xor(M, o, 64)); M2 = fmaxf(M2, __shfl_xor(M2, o, 64)); }
        sum = (m == -INFINITY) ? 0.f : sum * __expf(m - M);
        sum2 = (m2 == -INFINITY) ? 0.f : sum2 * __expf(m2 - M2);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) { sum += __shfl_xor(sum, o, 64); sum2 += __shfl_xor(sum2, o, 64); }
        if (lane == 0) { st[0][tl] = M; st[1][tl] = 1.f / sum; st[2][tl] = M2; st[3][tl] = row2 ? 1.f / sum2 : 0.f; }
    }
    __syncthreads();
    bf16* dst[4] = {out.hi + g * group_stride, out.lo + g * group_stride, out.dhi ? out.dhi + g * group_stride : nullptr,
                    out.dlo ? out.dlo + g * group_stride : nullptr};
    const int nparts = s2 ? 4 : 2;
    const int iend = min(L, (t0 / 256 + 1) * 256);
    // reading a 64 x 64 piece: thread (row tr of the piece, quarter sq) takes the columns 16 q + 4 sq + 0..3, q = 0..3, so that a row
    // is read as whole 64-byte runs and the transposed LDS writes of the four threads of a row fall into different banks;
    // writing it: thread (row tr of the transposed piece, 16 consecutive t from kc)
    const int tr = threadIdx.x >> 2, sq = threadIdx.x & 3, kc = sq * 16, t = t0 + tr;
    const float m = st[0][tr], inv = st[1][tr], m2 = st[2][tr], inv2 = st[3][tr];
    for (int i0 = 0; i0 < iend; i0 += 64) {
        if (i0 <= t0) {     // the piece holds entries on or left of the diagonal
            const float* src = s + (long long)t * L + i0 + 4 * sq;
            const float* src2 = s2 ? s2 + (long long)t * L + i0 + 4 * sq : nullptr;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4 v = *(const f4*)(src + 16 * q);
                f4 w = {0.f, 0.f, 0.f, 0.f};
                if (src2) w = *(const f4*)(src2 + 16 * q);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int il = 16 * q + 4 * sq + e, i = i0 + il;
                    const float a = i <= t ? __expf(v[e] - m) * inv : 0.f;
                    const bf16 ah = enc16(a, f16);
                    tp[0][il][tr] = ah;
                    tp[1][il][tr] = enc16(a - dec16(ah, f16), f16);
                    if (src2) {
                        const float da = a - (i <= t ? __expf(w[e] - m2) * inv2 : 0.f);
                        const bf16 dh = enc16(da, f16);
                        tp[2][il][tr] = dh;
                        tp[3][il][tr] = enc16(da - dec16(dh, f16), f16);
                    }
                }
            }
        } else {
            const bf16 zero = enc16(0.f, f16);
            for (int pt = 0; pt < nparts; ++pt)
#pragma unroll
                for (int e = 0; e < 16; ++e) tp[pt][kc + e][tr] = zero;
        }
        __syncthreads();
        {   // thread: row i0 + tr of the piece, 16 consecutive t from kc: two 16-byte chunks of a block row
            const long long col = (long long)r * L + t0 + kc;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const long long o = tboa_blocked_offset(i0 + tr, col + 8 * q, ldp >> 5);
                for (int pt = 0; pt < nparts; ++pt) *(uint4*)(dst[pt] + o) = *(const uint4*)&tp[pt][tr][kc + 8 * q];
            }
        }
        __syncthreads();
    }
}

// [B1 | B2^T] of a group -> the blocked 16-bit operand [B1_hi | B1_lo | B2^T_hi | B2^T_lo] (or [B1_hi | B1_lo] without B2):
// element (i, seg L + j).  B1 and B2^T arrive as `parts` partial sums (over subsets of the group's heads), fp32 row-major
// [parts][groups][L, L]; of the symmetric B1 only the 256-tiles on or below the diagonal are valid, the rest is taken from
// the mirrored tile through LDS.  One workgroup per 64 x 64 piece: thread (row, 16 consecutive columns).
__global__ __launch_bounds__(256) void bcat_kernel(const float* __restrict__ B1, const float* __restrict__ B2, int L, int parts, long long part_stride,
                                                   bf16* __restrict__ out, long long ldb, long long group_stride, int f16) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ float tt[64][65];
    const long long nn = (long long)L * L;
    const int g = blockIdx.z, i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    const int tr = threadIdx.x >> 2, c0 = (threadIdx.x & 3) * 16;
    bf16* o = out + g * group_stride;
    for (int which = 0; which < (B2 ? 2 : 1); ++which) {
        const float* src = (which ? B2 : B1) + g * nn;
        float v[16];
        if (which == 0 && (j0 >> 8) > (i0 >> 8)) {      // B1 above the diagonal tiles: the piece (j0, i0), transposed
            f4 acc[4] = {};
            for (int p = 0; p < parts; ++p)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] += *(const f4*)(src + p * part_stride + (long long)(j0 + tr) * L + i0 + c0 + 4 * q);
            __syncthreads();
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) tt[tr][c0 + 4 * q + e] = acc[q][e];
            __syncthreads();
#pragma unroll
            for (int e = 0; e < 16; ++e) v[e] = tt[c0 + e][tr];
        } else {
            f4 acc[4] = {};
            for (int p = 0; p < parts; ++p)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] += *(const f4*)(src + p * part_stride + (long long)(i0 + tr) * L + j0 + c0 + 4 * q);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) v[4 * q + e] = acc[q][e];
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            union { bf16 b[8]; uint4 u; } hi, lo;
#pragma unroll
            for (int k = 0; k < 8; ++k) { hi.b[k] = enc16(v[8 * q + k], f16); lo.b[k] = enc16(v[8 * q + k] - dec16(hi.b[k], f16), f16); }
            *(uint4*)(o + tboa_blocked_offset(i0 + tr, (2LL * which) * L + j0 + c0 + 8 * q, ldb >> 5)) = hi.u;
            *(uint4*)(o + tboa_blocked_offset(i0 + tr, (2LL * which + 1) * L + j0 + c0 + 8 * q, ldb >> 5)) = lo.u;
        }
    }
}

// largest |x| of a bf16 array, as the bits of a non-negative float (atomicMax on the integer); a NaN counts as infinity.
// Eight values per 16-byte load where the pointer allows it.
__global__ void absmax_bf16_kernel(const bf16* __restrict__ x, long long n, int* __restrict__ out) {
    float m = 0.f;
    auto take = [&](float v) { v = fabsf(v); m = (v > m || !(v == v)) ? (v == v ? v : INFINITY) : m; };
    const long long tid = blockIdx.x * (long long)blockDim.x + threadIdx.x, nth = (long long)gridDim.x * blockDim.x;
    const long long n8 = (((uintptr_t)x & 15) == 0) ? n / 8 : 0;
    for (long long i = tid; i < n8; i += nth) {
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        union { u4 u; bf16 b[8]; } v;
        v.u = __builtin_nontemporal_load((const u4*)x + i);
#pragma unroll
        for (int k = 0; k < 8; ++k) take(__bfloat162float(v.b[k]));
    }
    for (long long i = 8 * n8 + tid; i < n; i += nth) take(__bfloat162float(x[i]));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(out, __float_as_int(m));
}

// out = scale * sum_s partial[s] (fp64 accumulation); lower: only r >= c is read, the result is mirrored.
// vec (not with lower; n * n a multiple of 4, 16-byte aligned buffers): four consecutive elements per thread, the partial
// sums read once with 16-byte streaming loads.
__global__ void splitk_reduce_kernel(const float* __restrict__ part, int splits, int n, double scale, int lower, float* __restrict__ out, int vec) {
    const long long nn = (long long)n * n;
    if (vec) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < nn / 4; i += (long long)gridDim.x * blockDim.x) {
            double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
            for (int s = 0; s < splits; ++s) {
                const f4 v = __builtin_nontemporal_load((const f4*)(part + s * nn) + i);
                a0 += (double)v.x; a1 += (double)v.y; a2 += (double)v.z; a3 += (double)v.w;
            }
            const f4 o = {(float)(scale * a0), (float)(scale * a1), (float)(scale * a2), (float)(scale * a3)};
            ((f4*)out)[i] = o;
        }
        return;
    }
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < nn; i += (long long)gridDim.x * blockDim.x) {
        const int r = (int)(i / n), c = (int)(i % n);
        const long long src = (lower && c > r) ? (long long)c * n + r : i;
        double acc = 0.0;
        for (int s = 0; s < splits; ++s) acc += (double)part[s * nn + src];
        out[i] = (float)(scale * acc);
    }
}

// The same for a symmetric result whose partial sums hold the lower tiles only: tile pair (tr >= tc) per workgroup, the
// lower tile summed from coalesced reads and written with its mirror image through LDS.  vec (n a multiple of 64, 16-byte
// aligned buffers): off the diagonal a thread sums four consecutive columns from 16-byte streaming loads and writes four
// consecutive elements of a mirrored row.
__global__ __launch_bounds__(256) void splitk_reduce_lower_kernel(const float* __restrict__ part, int splits, int n, double scale,
                                                                  float* __restrict__ out, int vec) {
    __shared__ float t[64][65];
    const long long nn = (long long)n * n;
    int tr = (int)((sqrtf(8.f * (float)blockIdx.x + 1.f) - 1.f) * 0.5f);
    while ((long long)(tr + 1) * (tr + 2) / 2 <= (long long)blockIdx.x) ++tr;
    while ((long long)tr * (tr + 1) / 2 > (long long)blockIdx.x) --tr;
    const int tc = (int)(blockIdx.x - (long long)tr * (tr + 1) / 2);
    const int r0 = tr * 64, c0 = tc * 64;
    if (vec && tr != tc) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        for (int i = threadIdx.x; i < 64 * 16; i += 256) {
            const int r = i >> 4, c = (i & 15) * 4;
            const long long src = (long long)(r0 + r) * n + c0 + c;
            double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
            for (int s = 0; s < splits; ++s) {
                const f4 v = __builtin_nontemporal_load((const f4*)(part + s * nn + src));
                a0 += (double)v.x; a1 += (double)v.y; a2 += (double)v.z; a3 += (double)v.w;
            }
            const f4 o = {(float)(scale * a0), (float)(scale * a1), (float)(scale * a2), (float)(scale * a3)};
            *(f4*)(out + src) = o;
            t[r][c] = o.x; t[r][c + 1] = o.y; t[r][c + 2] = o.z; t[r][c + 3] = o.w;
        }
        __syncthreads();
        for (int i = threadIdx.x; i < 64 * 16; i += 256) {
            const int c = i >> 4, r = (i & 15) * 4;
            const f4 o = {t[r][c], t[r + 1][c], t[r + 2][c], t[r + 3][c]};
            *(f4*)(out + (long long)(c0 + c) * n + r0 + r) = o;
        }
        return;
    }
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int r = i >> 6, c = i & 63;
        float v = 0.f;
        if (r0 + r < n && c0 + c < n) {
            // on the diagonal tile the entries above the diagonal take their mirror image
            const long long src = (c0 + c > r0 + r) ? (long long)(c0 + c) * n + r0 + r : (long long)(r0 + r) * n + c0 + c;
            double acc = 0.0;
            for (int s = 0; s < splits; ++s) acc += (double)part[s * nn + src];
            v = (float)(scale * acc);
            out[(long long)(r0 + r) * n + c0 + c] = v;
        }
        t[r][c] = v;
    }
    if (tr == tc) return;
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int c = i >> 6, r = i & 63;
        if (r0 + r < n && c0 + c < n) out[(long long)(c0 + c) * n + r0 + r] = t[r][c];
    }
}

__global__ void bcast_heads_kernel(const double* __restrict__ src, float* __restrict__ dst, int rep, long long per, long long total) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const long long h = i / per, e = i % per;
        dst[i] = (float)src[(h / rep) * per + e];
    }
}

// out[row, :] = Min-Max fake-quant of in[row, :] (asymmetric, range extended to contain 0, a flat row takes [-1, 1]), one
// wavefront per row of n elements, everything in fp64 in the order of operations of the activation quantizer of Sec. 4.2:
// s = (hi - lo) / maxq, z = round(-lo / s), level = clamp(round(x / s) + z, 0, maxq), out = s (level - z).  In place is fine.
template <typename TI>
__global__ __launch_bounds__(256) void row_fakequant_f64_kernel(const TI* __restrict__ in, double* __restrict__ out, long long rows, int n, double maxq) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const TI* x = in + row * n; double* y = out + row * n;
    double lo = 0.0, hi = 0.0;
    for (int c = lane; c < n; c += 64) { const double v = (double)x[c]; lo = fmin(lo, v); hi = fmax(hi, v); }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { lo = fmin(lo, __shfl_xor(lo, o, 64)); hi = fmax(hi, __shfl_xor(hi, o, 64)); }
    if (lo == hi) { lo = -1.0; hi = 1.0; }
    const double s = (hi - lo) / maxq, z = rint(-lo / s);
    for (int c = lane; c < n; c += 64) {
        const double v = (double)x[c];
        const double q = fmin(fmax(rint(v / s) + z, 0.0), maxq);
        y[c] = s * (q - z);
    }
}

// Row pitches that are multiples of a few KB put every row of a tile into the same memory channel; 256 extra
// elements per row spread them (measured: +10..20 % on the GEMMs).
constexpr int PADE = 256;

inline unsigned g1(long long n) { long long g = (n + 255) / 256; return (unsigned)(g < 1 ? 1 : (g > 32768 ? 32768 : g)); }

struct Dims {
    tboa_ctx* ctx; const tboa_attn_desc* d;
    int T, dm, Hq, Hkv, dh, L, S, rep, dq, dkv;
    int f16;      // the 16-bit operands of the W_V / W_O chains are IEEE half (else bf16)
};

Dims dims_of(tboa_ctx* ctx, const tboa_attn_desc* d) {
    return Dims{ctx, d, d->n_seqs * d->seq_len, d->d_model, d->n_q_heads, d->n_kv_heads, d->head_dim, d->seq_len, d->n_seqs,
                d->n_q_heads / d->n_kv_heads, d->n_q_heads * d->head_dim, d->n_kv_heads * d->head_dim, 0};
}

// Q^ and K^ (the three-segment operands of the score products) are kept per (sequence, head) in 16 x 32 blocks when the
// shapes allow it: whole 1 KB blocks instead of 64-byte row pieces at a pitch of all heads
bool qk_blocked(const Dims& D) { return D.L % 16 == 0 && (3 * D.dh) % 32 == 0; }

int pick_splits(int n_seqs) {
    for (int s = 16; s > 1; --s) if (n_seqs % s == 0) return s;
    return 1;
}

// Whether the activations fit IEEE half (|x| < 2^15, finite): one reduction over each array, one read-back.
int fits_half(tboa_ctx* ctx, const bf16* X, const bf16* X_fp, long long n, int* fits, float* amax = nullptr) {
    int* w = ctx->d_status + 5;
    TB_HIP(ctx, hipMemsetAsync(w, 0, sizeof(int), ctx->stream));
    hipLaunchKernelGGL(absmax_bf16_kernel, dim3(2048), dim3(256), 0, ctx->stream, X, n, w);
    if (X_fp) hipLaunchKernelGGL(absmax_bf16_kernel, dim3(2048), dim3(256), 0, ctx->stream, X_fp, n, w);
    TB_KERNEL_CHECK(ctx);
    TB_HIP(ctx, hipMemcpyAsync(ctx->h_status + 5, w, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    TB_HIP(ctx, hipStreamSynchronize(ctx->stream));
    float m; memcpy(&m, ctx->h_status + 5, sizeof(float));
    *fits = (m < 32768.f) ? 1 : 0;
    if (amax) *amax = m;
    return 0;
}

int transpose(const Dims& D, const bf16* in, const bf16* in2, long long ld_in, int rows, int cols, bf16* out, bf16* hi, bf16* lo, long long ld_out,
              int blocked = 0, int f16 = 0) {
    auto al = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
    const int vec = ld_in % 8 == 0 && ld_out % 8 == 0 && al(in) && al(in2) && al(out) && al(hi) && al(lo);
    hipLaunchKernelGGL(transpose_kernel, dim3((cols + 63) / 64, (rows + 63) / 64), dim3(256), 0, D.ctx->stream, in, in2, ld_in, rows, cols,
                       out, hi, lo, ld_out, blocked, vec, f16);
    TB_HIP(D.ctx, hipGetLastError());
    return 0;
}

GemmBf16 nt(int M, int N, int K, float alpha, const bf16* A, long long lda, const bf16* B, long long ldb, void* C, long long ldc,
            int c_dtype, int accumulate, int flags) {
    GemmBf16 g{};
    g.M = M; g.N = N; g.K = K; g.alpha = alpha; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
    // The Hessian builds have the GPU to themselves, and most of their products have short contractions (a sequence, a
    // head): the persistent kernel, which hides the ring fill and the tile's write-out, is the default here; the callers
    // with long contractions (gram_splitk, the sums over a chunk of sequences) clear the flag.
    g.c_dtype = c_dtype; g.accumulate = accumulate; g.flags = flags | TBOA_GEMM_PERSISTENT; g.batch = 1; g.tag = TBOA_PROF_PROJ;
    return g;
}

// out[n, n] = scale * sum over the operand pairs p of A_p B_p^T, with the contraction over all T tokens split into `splits`
// chunks (an exact-to-16-bit (hi, lo) operand takes part as several pairs: hi.hi + lo.hi + hi.lo)
struct GramPair { const bf16* A; const bf16* B; };
int gram_splitk(tboa_ctx* ctx, int splits, int n, int npairs, const GramPair* pairs, long long ld, int K, double scale, int lower,
                float* part, float* out, int f16 = 0) {
    const int Kc = K / splits;
    GemmBf16 g = nt(n, n, Kc, 1.f, pairs[0].A, ld, pairs[0].B, ld, part, n, TBOA_F32, 0, (lower ? TBOA_GEMM_LOWER : 0) | (f16 ? TBOA_GEMM_F16 : 0));
    g.tag = TBOA_PROF_GRAM; g.flags &= ~TBOA_GEMM_PERSISTENT;
    g.batch = splits; g.strideA = Kc; g.strideB = Kc; g.strideC = (long long)n * n;
    if (lower) TB_TRY(launch_fill_f32(ctx, part, (int64_t)splits * n * n, 0.f));
    for (int p = 0; p < npairs; ++p) {
        g.A = pairs[p].A; g.B = pairs[p].B; g.accumulate = p ? 1 : 0;
        TB_TRY(gemm_bf16_nt(ctx, g));
    }
    const bool aligned16 = (((uintptr_t)part | (uintptr_t)out) & 15) == 0;
    const int vec = (!lower && aligned16 && ((long long)n * n) % 4 == 0) ? 1 : 0;
    if (lower) {
        const long long nt = (n + 63) / 64;
        hipLaunchKernelGGL(splitk_reduce_lower_kernel, dim3((unsigned)(nt * (nt + 1) / 2)), dim3(256), 0, ctx->stream, part, splits, n, scale, out,
                           (n % 64 == 0 && aligned16) ? 1 : 0);
    } else
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(g1((long long)n * n / (vec ? 4 : 1))), dim3(256), 0, ctx->stream, part, splits, n, scale, lower, out, vec);
    TB_HIP(ctx, hipGetLastError());
    return 0;
}
int gram_splitk(tboa_ctx* ctx, int splits, int n, const bf16* A, const bf16* A_lo, const bf16* B, long long ld, int K, double scale, int lower,
                float* part, float* out) {
    const GramPair pairs[2] = {{A, B}, {A_lo, B}};
    return gram_splitk(ctx, splits, n, A_lo ? 2 : 1, pairs, ld, K, scale, lower, part, out);
}

// Q^ [rows, Hq, 3 dh] and K^ [rows, Hkv, 3 dh] of `rows` tokens Xr [rows, d]; weights as one, two or three bf16 terms.
// amax_q, amax_k (both or neither; blocked operands of whole sequences only): one device word per sequence of the chunk each;
// the pairs are then scaled IEEE half values and the words say by how much (see QkScale), else unscaled bf16.
int project_qk(const Dims& D, const bf16* Xr, int rows, const bf16* Wq, const bf16* Wq_lo, const bf16* Wk, const bf16* Wk_lo,
               float* Qf, float* Kf, bf16* Qh, bf16* Kh, const float* q_scale = nullptr, const float* k_scale = nullptr,
               int* amax_q = nullptr, int* amax_k = nullptr, const bf16* Wq_lo2 = nullptr, const bf16* Wk_lo2 = nullptr) {
    // (the smallest term first: the sum then rounds where the largest term does)
    const bf16* tq[3] = {Wq_lo2, Wq_lo, Wq}; const bf16* tk[3] = {Wk_lo2, Wk_lo, Wk};
    int first = 1;
    for (const bf16* w : tq) if (w) { TB_TRY(gemm_bf16_nt(D.ctx, nt(rows, D.dq, D.dm, 1.f, Xr, D.dm, w, D.dm, Qf, D.dq, TBOA_F32, first ? 0 : 1, 0))); first = 0; }
    first = 1;
    for (const bf16* w : tk) if (w) { TB_TRY(gemm_bf16_nt(D.ctx, nt(rows, D.dkv, D.dm, 1.f, Xr, D.dm, w, D.dm, Kf, D.dkv, TBOA_F32, first ? 0 : 1, 0))); first = 0; }
    if (amax_q) {
        if (!amax_k || !qk_blocked(D) || D.dh % 32 || rows % D.L) return tboa_fail(D.ctx, TBOA_EINVAL, "project_qk: half operands need blocked whole sequences");
        const int ns = rows / D.L;
        TB_TRY(launch_fill_f32(D.ctx, (float*)amax_q, ns, -1.f));       // any negative word: the bits of the largest magnitude replace it
        TB_TRY(launch_fill_f32(D.ctx, (float*)amax_k, ns, -1.f));
        hipLaunchKernelGGL(amax_seq_kernel, dim3(256, ns), dim3(256), 0, D.ctx->stream, Qf, q_scale, D.L, D.dq, amax_q);
        hipLaunchKernelGGL(amax_seq_kernel, dim3(256, ns), dim3(256), 0, D.ctx->stream, Kf, k_scale, D.L, D.dkv, amax_k);
    }
    hipLaunchKernelGGL(split3_kernel, dim3(g1((long long)rows * D.dq)), dim3(256), 0, D.ctx->stream, Qf, q_scale, Qh, (long long)rows, D.dq, D.dh, 0,
                       qk_blocked(D) ? D.L : 0, amax_q);
    hipLaunchKernelGGL(split3_kernel, dim3(g1((long long)rows * D.dkv)), dim3(256), 0, D.ctx->stream, Kf, k_scale, Kh, (long long)rows, D.dkv, D.dh, 1,
                       qk_blocked(D) ? D.L : 0, amax_k);
    TB_HIP(D.ctx, hipGetLastError());
    return 0;
}

// scaled scores Q_h K_g^T / sqrt(d_h) of all heads of local sequence sl -> Sc [Hq, L, L] (lower tiles when causal)
int scores(const Dims& D, const bf16* Qh, const bf16* Kh, int sl, float* Sc) {
    const int L = D.L, dh3 = 3 * D.dh;
    GemmBf16 g = nt(L, L, dh3, (float)(1.0 / sqrt((double)D.dh)), Qh + (long long)sl * L * D.Hq * dh3, (long long)D.Hq * dh3,
                    Kh + (long long)sl * L * D.Hkv * dh3, (long long)D.Hkv * dh3, Sc, L, TBOA_F32, 0, D.d->causal ? TBOA_GEMM_LOWER : 0);
    g.batch = D.Hq; g.batch_inner = D.rep; g.tag = TBOA_PROF_SCORES;
    g.strideA = (long long)D.rep * dh3; g.strideA2 = dh3; g.strideB = dh3; g.strideB2 = 0;
    if (qk_blocked(D)) {     // one blocked [L, 3 dh] matrix per (sequence, head)
        g.flags |= TBOA_GEMM_A_TILED | TBOA_GEMM_B_TILED; g.lda = dh3; g.ldb = dh3;
        g.strideA = (long long)D.rep * L * dh3; g.strideA2 = (long long)L * dh3; g.strideB = (long long)L * dh3;
    }
    g.strideC = (long long)D.rep * L * L; g.strideC2 = (long long)L * L;
    return gemm_bf16_nt(D.ctx, g);
}

// Both score matrices of a sequence (the quantized-input path and the full-precision path).  With one query head per KV
// head the two products are one launch whose outer batch index is the path: 2 x 36 x H tiles fill the 256 CUs evenly
// where 36 x H leave the last round half empty.  (The path stride is the distance between the two buffers.)
int scores_pair(const Dims& D, const bf16* Qh, const bf16* Kh, const bf16* Qhf, const bf16* Khf, int sl, float* Sc, float* Scf) {
    const long long dq = Qhf - Qh, dk = Khf - Kh, dc = Scf - Sc;
    if (D.rep != 1 || dq % 8 || dk % 8 || dc % 4) {
        TB_TRY(scores(D, Qh, Kh, sl, Sc));
        return scores(D, Qhf, Khf, sl, Scf);
    }
    const int L = D.L, dh3 = 3 * D.dh;
    GemmBf16 g = nt(L, L, dh3, (float)(1.0 / sqrt((double)D.dh)), Qh + (long long)sl * L * D.Hq * dh3, (long long)D.Hq * dh3,
                    Kh + (long long)sl * L * D.Hkv * dh3, (long long)D.Hkv * dh3, Sc, L, TBOA_F32, 0, D.d->causal ? TBOA_GEMM_LOWER : 0);
    g.batch = 2 * D.Hq; g.batch_inner = D.Hq; g.tag = TBOA_PROF_SCORES;
    g.strideA = dq; g.strideA2 = dh3; g.strideB = dk; g.strideB2 = dh3;
    if (qk_blocked(D)) {
        g.flags |= TBOA_GEMM_A_TILED | TBOA_GEMM_B_TILED; g.lda = dh3; g.ldb = dh3;
        g.strideA2 = (long long)L * dh3; g.strideB2 = (long long)L * dh3;
    }
    g.strideC = dc; g.strideC2 = (long long)L * L;
    return gemm_bf16_nt(D.ctx, g);
}

// probabilities in 16 x 32 blocks (per head) when `blocked`: see blocked_inputs
int softmax(const Dims& D, const float* Sc, const float* Sc2, bf16* P, long long ldp, int hi2col, int locol, int dcol, int blocked = 0, int pair2 = 0) {
    if (D.L % 4 == 0 && D.L <= 2048 && ldp % 4 == 0 && dcol % 4 == 0)
        hipLaunchKernelGGL(softmax_bf16_regs_kernel<8>, dim3((D.L + 3) / 4, D.Hq), dim3(256), 0, D.ctx->stream, Sc, Sc2, D.L, D.d->causal, P,
                           ldp, (long long)D.L * ldp, hi2col, locol, dcol, blocked, D.f16, pair2);
    else if (blocked) return tboa_fail(D.ctx, TBOA_EINVAL, "softmax: blocked probabilities need the in-register kernel");
    else
        hipLaunchKernelGGL(softmax_bf16_kernel, dim3((D.L + 3) / 4, D.Hq), dim3(256), 0, D.ctx->stream, Sc, Sc2, D.L, D.d->causal, P, ldp,
                           (long long)D.L * ldp, hi2col, locol, dcol, D.f16, pair2);
    TB_HIP(D.ctx, hipGetLastError());
    return 0;
}

// The transposed activations and the probabilities are operands of the A X products only: they are kept in the GEMM's
// 16 x 32 blocks when the shapes allow (whole blocks, the in-register softmax)
bool blocked_inputs(const Dims& D) {
    return D.L % 32 == 0 && D.L <= 2048 && D.dm % 16 == 0;
}

// The form of the W_V Hessian that works on L x L Gram matrices of the probabilities (see build_hessians_bf16): needs
// whole 256-tiles and causal probabilities.  Other shapes take the per-head products.
bool summed_form(const Dims& D) {
    return D.d->causal && D.L % 256 == 0 && D.dm % 256 == 0;
}

int check_bf16_dims(const Dims& D) {
    if (D.L % 8 || D.dm % 8 || D.dh % 8)
        return tboa_fail(D.ctx, TBOA_EINVAL, "bf16 Hessian build needs seq_len, d_model and head_dim to be multiples of 8");
    return 0;
}

// H_in and R of W_V for bf16 inputs (Table 1: X A_h^T A_h X^T, summed over the sequences and the query heads of the KV group).
//
// Summed form (summed_form: every named configuration):  sum_{h in g} (A_h X_s)^T (A_h X_s) = X_s^T (sum_h A_h^T A_h) X_s, so
// the sum over the heads of a group is taken on L x L matrices and the products that are d wide run once per (sequence,
// group), with the exact input X_s as one operand:
//     B1 = sum_h A_h^T A_h,   B2^T = sum_h A_h^T (A_h - A~_h)         [L, L] per group, from transposed probabilities
//     T1 = B1 X_s,   Z = B1 dX_s + B2^T X~_s                            [L, d]
//     H_in^V[g] += T1^T X_s,   R_v[g] += alpha Z^T X_s                 summed over a chunk of sequences per launch
// since sum_h (A_h X - A~_h X~)^T (A_h X) = sum_h (A_h dX + (A_h - A~_h) X~)^T A_h X.  Every intermediate (A, A - A~, B1, B2,
// T1, Z) is carried as an exact-to-twice-the-mantissa (hi, lo) pair of 16-bit values and every product accumulates
// hi.hi + lo.hi + hi.lo in fp32, so the result is fp32-grade (measured against fp64: 1e-6 of the diagonal).  A_h^T has
// zeros above its diagonal, so the contractions over the tokens t start at the tile of max(i, j) (TBOA_GEMM_KLO).
//
// Per-head form (shapes without whole 256-tiles, or no causal mask):  Y_h = A_h X_s per (sequence, head), H_in^V += Y^T Y,
// R_v += alpha dY^T Y with dY = A dX + (A - A~) X~; probabilities and Y are single 16-bit values there (1e-4-grade).
int build_hessians_bf16(tboa_ctx* ctx, const tboa_attn_desc* d, const bf16* X, const bf16* X_fp, const bf16* Wq, const bf16* Wk,
                        const bf16* Wo, float* Hin_qk, float* R_qk, float* Hout_q, float* Hout_k, float* Hin_v, float* R_v, float* Hout_v,
                        bf16* fp_cache) {
    Dims D = dims_of(ctx, d);
    TB_TRY(check_bf16_dims(D));
    const int T = D.T, dm = D.dm, Hq = D.Hq, Hkv = D.Hkv, dh = D.dh, L = D.L, dq = D.dq, dkv = D.dkv, rep = D.rep;
    const bool fp = X_fp != nullptr, rv = fp && R_v;
    const bool grouped = summed_form(D);
    const bool fused = grouped && qk_blocked(D) && attn_probs_t_supported(D.L, D.dh);     // no score matrices in memory
    int G = d->seq_chunk > 0 ? d->seq_chunk : 8; if (G > D.S) G = D.S;
    // segments of P / of the transposed chunk ([X | dX | X~]; summed form: every one twice, for the (hi, lo) operands it meets)
    const int nsg = rv ? 2 : 1, nsx = (grouped ? 2 : 1) * (rv ? 3 : 1), splits = pick_splits(D.S);
    const long long dd = (long long)dm * dm, hh = (long long)dh * dh, TP = (long long)T + PADE;
    // summed form: pitches of the transposed probabilities, of [B1_hi | B1_lo | B2^T_hi | B2^T_lo], of the chunk buffers
    const long long ldpt = (long long)rep * L + PADE, ldbc = (rv ? 4LL : 2LL) * L + PADE, ldg = (long long)G * L + PADE;
    // summed form: the L x L Gram matrices of a group are built as `parts` partial sums over subsets of its heads (added up
    // where they are split into 16-bit operands): the tile at the origin contracts over all L tokens of every head, the tile at
    // the far corner over 256, so with few batch entries the longest tile alone would set the time of the launch
    const int parts = (Hkv < 32 && rep % 2 == 0) ? 2 : 1;
    bf16 *XT, *dXh, *dXl, *Qh, *Kh, *Qhf, *Khf, *P, *XcT, *YT, *dYT;
    bf16 *Bcat = nullptr, *XgT = nullptr, *XgTh = nullptr, *YTl = nullptr, *dYTl = nullptr;
    PtOut pt{nullptr, nullptr, nullptr, nullptr};
    float *part, *Qf, *Kf, *Sc, *Scf, *B1f = nullptr, *B2f = nullptr;
    int* amx;      // [q | k | q~ | k~] x G: largest magnitudes of the chunk's projections, per sequence (see QkScale)
    double *Hin64, *Wq64, *Wk64, *Wo64, *Tq, *Tk, *Ho;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        XT = ar.get<bf16>((size_t)dm * TP);
        dXh = fp ? ar.get<bf16>((size_t)dm * TP) : nullptr; dXl = fp ? ar.get<bf16>((size_t)dm * TP) : nullptr;
        part = ar.get<float>((size_t)splits * dd);
        Qf = ar.get<float>((size_t)G * L * dq); Kf = ar.get<float>((size_t)G * L * dkv);
        Qh = ar.get<bf16>((size_t)G * L * dq * 3); Kh = ar.get<bf16>((size_t)G * L * dkv * 3);
        Qhf = rv ? ar.get<bf16>((size_t)G * L * dq * 3) : nullptr; Khf = rv ? ar.get<bf16>((size_t)G * L * dkv * 3) : nullptr;
        Sc = fused ? nullptr : ar.get<float>((size_t)Hq * L * L); Scf = (rv && !fused) ? ar.get<float>((size_t)Hq * L * L) : nullptr;
        amx = ar.get<int>((size_t)4 * G);
        XcT = ar.get<bf16>((size_t)dm * (G * nsx * L + PADE));
        if (grouped) {
            P = nullptr;
            pt.hi = ar.get<bf16>((size_t)Hkv * L * ldpt); pt.lo = ar.get<bf16>((size_t)Hkv * L * ldpt);
            pt.dhi = rv ? ar.get<bf16>((size_t)Hkv * L * ldpt) : nullptr; pt.dlo = rv ? ar.get<bf16>((size_t)Hkv * L * ldpt) : nullptr;
            B1f = ar.get<float>((size_t)parts * Hkv * L * L); B2f = rv ? ar.get<float>((size_t)parts * Hkv * L * L) : nullptr;
            Bcat = ar.get<bf16>((size_t)Hkv * L * ldbc);
            XgT = ar.get<bf16>((size_t)dm * ldg); XgTh = ar.get<bf16>((size_t)dm * ldg);
            YT = ar.get<bf16>((size_t)Hkv * dm * ldg); YTl = ar.get<bf16>((size_t)Hkv * dm * ldg);
            dYT = rv ? ar.get<bf16>((size_t)Hkv * dm * ldg) : nullptr; dYTl = rv ? ar.get<bf16>((size_t)Hkv * dm * ldg) : nullptr;
        } else {
            P = ar.get<bf16>((size_t)Hq * L * (nsg * L + PADE));
            YT = ar.get<bf16>((size_t)Hkv * dm * (rep * G * L + PADE)); dYT = rv ? ar.get<bf16>((size_t)Hkv * dm * (rep * G * L + PADE)) : nullptr;
        }
        Hin64 = ar.get<double>((size_t)dd); Wq64 = ar.get<double>((size_t)dq * dm); Wk64 = ar.get<double>((size_t)dkv * dm);
        Wo64 = ar.get<double>((size_t)dm * dq); Tq = ar.get<double>((size_t)dq * dm); Tk = ar.get<double>((size_t)dkv * dm);
        Ho = ar.get<double>((size_t)Hkv * hh);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    hipStream_t st = ctx->stream;
    // ---- H_in and R for W_Q / W_K
    if (Hin_qk) {
    TB_TRY(transpose(D, X, fp ? X_fp : nullptr, dm, T, dm, XT, fp ? dXh : nullptr, dXl, TP));
    TB_TRY(gram_splitk(ctx, splits, dm, XT, nullptr, XT, TP, T, 1.0, 1, part, Hin_qk));
    if (fp && R_qk) TB_TRY(gram_splitk(ctx, splits, dm, dXh, dXl, XT, TP, T, d->alpha, 0, part, R_qk));
    // ---- H_out: K_g^T K_g = W_K,g H_in W_K,g^T ; sum_h Q_h^T Q_h ; sum_h W_out,h^T W_out,h   (fp64)
    TB_TRY(launch_cvt_f32_to_f64(ctx, Hin_qk, Hin64, dd));
    TB_TRY(launch_cvt_to_f64(ctx, Wq, TBOA_BF16, Wq64, (int64_t)dq * dm));
    TB_TRY(launch_cvt_to_f64(ctx, Wk, TBOA_BF16, Wk64, (int64_t)dkv * dm));
    {
        GemmF64 a{};
        a.M = dq; a.N = dm; a.K = dm; a.alpha = 1.0; a.beta = 0.0; a.A = Wq64; a.sam = dm; a.sak = 1; a.B = Hin64; a.sbk = dm; a.sbn = 1;
        a.C = Tq; a.ldc = dm; a.batch = 1;
        TB_TRY(gemm_f64(ctx, a));
        a.M = dkv; a.A = Wk64; a.C = Tk;
        TB_TRY(gemm_f64(ctx, a));
        GemmF64 b{};   // per KV head: Tk_g Wk_g^T
        b.M = dh; b.N = dh; b.K = dm; b.alpha = 1.0; b.beta = 0.0; b.A = Tk; b.sam = dm; b.sak = 1; b.B = Wk64; b.sbk = 1; b.sbn = dm;
        b.C = Ho; b.ldc = dh; b.batch = Hkv; b.strideA = (long long)dh * dm; b.strideB = b.strideA; b.strideC = hh;
        TB_TRY(gemm_f64(ctx, b));
        hipLaunchKernelGGL(bcast_heads_kernel, dim3(g1(Hq * hh)), dim3(256), 0, st, Ho, Hout_q, rep, hh, Hq * hh);
        for (int r = 0; r < rep; ++r) {   // sum over the query heads of a group
            b.A = Tq + (long long)r * dh * dm; b.B = Wq64 + (long long)r * dh * dm; b.beta = r ? 1.0 : 0.0;
            b.strideA = (long long)rep * dh * dm; b.strideB = b.strideA;
            TB_TRY(gemm_f64(ctx, b));
        }
        hipLaunchKernelGGL(bcast_heads_kernel, dim3(g1(Hkv * hh)), dim3(256), 0, st, Ho, Hout_k, 1, hh, Hkv * hh);
        TB_KERNEL_CHECK(ctx);
    }
    }
    if (Hout_v) {
        TB_TRY(launch_cvt_to_f64(ctx, Wo, TBOA_BF16, Wo64, (int64_t)dm * dq));
        GemmF64 c{};   // W_out,h^T W_out,h, W_out,h = Wo[:, h dh : (h+1) dh]
        c.M = dh; c.N = dh; c.K = dm; c.alpha = 1.0; c.sam = 1; c.sak = dq; c.sbk = dq; c.sbn = 1; c.C = Ho; c.ldc = dh;
        c.batch = Hkv; c.strideA = (long long)rep * dh; c.strideB = c.strideA; c.strideC = hh;
        for (int r = 0; r < rep; ++r) {
            c.A = Wo64 + (long long)r * dh; c.B = c.A; c.beta = r ? 1.0 : 0.0;
            TB_TRY(gemm_f64(ctx, c));
        }
        hipLaunchKernelGGL(bcast_heads_kernel, dim3(g1(Hkv * hh)), dim3(256), 0, st, Ho, Hout_v, 1, hh, Hkv * hh);
        TB_KERNEL_CHECK(ctx);
    }
    // ---- H_in (and R) of W_V
    if (!Hin_v) return 0;
    float xmax = 0.f;
    TB_TRY(fits_half(ctx, X, rv ? X_fp : nullptr, (long long)T * dm, &D.f16, &xmax));
    // the Gram sums of the probabilities reach rep L where every query attends to one token (entry (i, i) of sum_h A_h^T A_h
    // is at most the number of (head, query) pairs): beyond the range of half they are carried as bf16 pairs
    if ((long long)rep * L >= 60000) D.f16 = 0;
    const int hf = D.f16 ? TBOA_GEMM_F16 : 0;
    // Summed form with half operands: T1 = B1 X and Z leave their products as pairs of halves (22 bits; as pairs of bf16, 16
    // bits, their rounding was what limited H_in^V), so the last products read a half copy of X^T (exact: bf16 has fewer
    // bits).  |T1| <= (row sum of B1) max|X| <= rep L max|X| and |Z| <= 3 times that (B1 dX + B2^T X~, |dX| <= 2 max, row sums of
    // |B2| <= 2 rep L): the products scale their results by a power of two that brings this bound under 2^15, and store the
    // low parts times 2^11 (the low part of a half is at most 2^-12 of it: no overflow, and normal numbers wherever the
    // high part is above 2^-13); the last products take the factors back out.
    const bool half_y = grouped && D.f16;
    int ey = 0, ez = 0;
    if (half_y) {
        const double bound = (double)rep * L * (xmax > 0.f ? xmax : 1.f);
        while (ldexp(bound, -ey) >= 32768.0) ++ey;
        ez = ey + 2;
    }
    TB_TRY(launch_fill_f32(ctx, Hin_v, (int64_t)Hkv * dd, 0.f));
    if (rv) TB_TRY(launch_fill_f32(ctx, R_v, (int64_t)Hkv * dd, 0.f));
    const int cflag = d->causal ? TBOA_GEMM_CAUSAL_K : 0;
    const bool blocked = dm % 256 == 0 && L % 256 == 0;
    const int bin = grouped ? 1 : blocked_inputs(D);      // (the grouped form has whole blocks by its own conditions)
    for (int s0 = 0; s0 < D.S; s0 += G) {
        const int Gc = (D.S - s0 < G) ? D.S - s0 : G;
        const long long t0 = (long long)s0 * L;
        const long long ldx = (long long)Gc * nsx * L + PADE, ky = (long long)rep * Gc * L, ldy = ky + PADE, ldp = (long long)nsg * L + PADE;
        // the fused kernel takes scaled half operands (22 significant bits in the scores instead of 16); the GEMM path bf16 pairs
        int *aq = fused ? amx : nullptr, *ak = fused ? amx + G : nullptr, *aqf = fused ? amx + 2 * G : nullptr, *akf = fused ? amx + 3 * G : nullptr;
        TB_TRY(project_qk(D, X + t0 * dm, Gc * L, Wq, nullptr, Wk, nullptr, Qf, Kf, Qh, Kh, nullptr, nullptr, aq, ak));
        if (rv && fp_cache) {   // the caller keeps the full-precision projections of all tokens: written in place, their words behind them
            Qhf = fp_cache + t0 * dq * 3; Khf = fp_cache + (long long)T * dq * 3 + t0 * dkv * 3;
            int* words = (int*)(fp_cache + (long long)T * (dq + dkv) * 3);
            if (fused) { aqf = words + s0; akf = words + D.S + s0; }
            else if (s0 == 0) TB_TRY(launch_fill_f32(ctx, (float*)words, 2LL * D.S, -1.f));      // negative words: bf16 pairs
        }
        if (rv) TB_TRY(project_qk(D, X_fp + t0 * dm, Gc * L, Wq, nullptr, Wk, nullptr, Qf, Kf, Qhf, Khf, nullptr, nullptr, aqf, akf));
        const long long is = bin ? 16 : 1;      // a column offset c into a blocked matrix is the pointer offset 16 c
        for (int sl = 0; sl < Gc; ++sl) {   // XcT[:, sl, :, :] = X_s^T | (X_s - X~_s)^T | X~_s^T
            const bf16* xs = X + (t0 + (long long)sl * L) * dm;
            bf16* o = XcT + is * sl * nsx * L;
            if (grouped) {      // [X | X | dX | dX | X~ | X~], and X_s^T once more as bf16 (the exact input), the chunk's sequences side by side
                const bf16* xf = rv ? X_fp + (t0 + (long long)sl * L) * dm : nullptr;
                for (int c = 0; c < 2; ++c) {
                    TB_TRY(transpose(D, xs, xf, dm, L, dm, o + 16LL * c * L, rv ? o + 16LL * (2 + c) * L : nullptr, nullptr, ldx, 1, D.f16));
                    if (rv) TB_TRY(transpose(D, xf, nullptr, dm, L, dm, o + 16LL * (4 + c) * L, nullptr, nullptr, ldx, 1, D.f16));
                }
                TB_TRY(transpose(D, xs, nullptr, dm, L, dm, XgT + 16LL * sl * L, nullptr, nullptr, ldg, 1, 0));
                if (half_y) TB_TRY(transpose(D, xs, nullptr, dm, L, dm, XgTh + 16LL * sl * L, nullptr, nullptr, ldg, 1, 1));
            } else if (!rv) TB_TRY(transpose(D, xs, nullptr, dm, L, dm, o, nullptr, nullptr, ldx, bin, D.f16));
            else {
                const bf16* xf = X_fp + (t0 + (long long)sl * L) * dm;
                TB_TRY(transpose(D, xs, xf, dm, L, dm, o, o + is * L, nullptr, ldx, bin, D.f16));
                TB_TRY(transpose(D, xf, nullptr, dm, L, dm, o + is * 2 * L, nullptr, nullptr, ldx, bin, D.f16));
            }
        }
        if (grouped) {
            const int tiled = TBOA_GEMM_A_TILED | TBOA_GEMM_B_TILED;
            for (int sl = 0; sl < Gc; ++sl) {
                if (fused) {       // scores and softmax in one kernel, nothing of the scores stored
                    const long long qo = (long long)sl * Hq * L * 3 * dh, ko = (long long)sl * Hkv * L * 3 * dh;
                    const QkScale qs{aq + sl, ak + sl, rv ? aqf + sl : nullptr, rv ? akf + sl : nullptr};
                    TB_TRY(attn_probs_t(ctx, Qh + qo, Kh + ko, rv ? Qhf + qo : nullptr, rv ? Khf + ko : nullptr, L, Hq, rep, dh, pt, ldpt,
                                        (long long)L * ldpt, D.f16, qs));
                } else {
                    if (rv) TB_TRY(scores_pair(D, Qh, Kh, Qhf, Khf, sl, Sc, Scf));
                    else TB_TRY(scores(D, Qh, Kh, sl, Sc));
                    hipLaunchKernelGGL(softmax_t_kernel, dim3(L / 64, Hq), dim3(256), 0, st, Sc, rv ? Scf : nullptr, L, rep, pt, ldpt,
                                       (long long)L * ldpt, D.f16);
                    TB_KERNEL_CHECK(ctx);
                }
                // B1 = sum_h A_h^T A_h and B2^T = sum_h A_h^T (A_h - A~_h): contraction over (head of the group, t >= max(i, j)) and
                // over the three products of (hi, lo) parts, in one pass.  B1 is symmetric: only its tiles on or below the diagonal
                // (half probabilities from the fused kernel carry ATTN_PROBS_HALF_SCALE each)
                const float pa = (fused && D.f16) ? 1.f / (ATTN_PROBS_HALF_SCALE * ATTN_PROBS_HALF_SCALE) : 1.f;
                GemmBf16 b = nt(L, L, 3 * (rep / parts) * L, pa, pt.hi, ldpt, pt.hi, ldpt, B1f, L, TBOA_F32, 0, tiled | TBOA_GEMM_KLO | TBOA_GEMM_LOWER | hf);
                b.kseg = L; b.batch = Hkv * parts; b.batch_inner = parts; b.tag = TBOA_PROF_ATA;
                b.strideA = (long long)L * ldpt; b.strideA2 = 16LL * (rep / parts) * L; b.strideB = b.strideA; b.strideB2 = b.strideA2;
                b.strideC = (long long)L * L; b.strideC2 = (long long)Hkv * L * L;
                b.nterms = 3;
                b.termA[0] = pt.hi; b.termA[1] = pt.lo; b.termA[2] = pt.hi;
                b.termB[0] = pt.hi; b.termB[1] = pt.hi; b.termB[2] = pt.lo;
                TB_TRY(gemm_bf16_nt(ctx, b));
                if (rv) {
                    b.flags &= ~TBOA_GEMM_LOWER; b.C = B2f; b.B = pt.dhi;
                    b.termB[0] = pt.dhi; b.termB[1] = pt.dhi; b.termB[2] = pt.dlo;
                    TB_TRY(gemm_bf16_nt(ctx, b));
                }
                hipLaunchKernelGGL(bcat_kernel, dim3(L / 64, L / 64, Hkv), dim3(256), 0, st, B1f, B2f, L, parts, (long long)Hkv * L * L, Bcat, ldbc,
                                   (long long)L * ldbc, D.f16);
                TB_KERNEL_CHECK(ctx);
                // T1^T = [X_s^T | X_s^T] [B1_hi | B1_lo]^T and Z^T = [dX_s^T | dX_s^T | X~_s^T | X~_s^T] [B1_hi | B1_lo | B2^T_hi | B2^T_lo]^T,
                // each left as a (hi, lo) pair: scaled halves (see half_y above), or bf16
                GemmBf16 y = nt(dm, L, 2 * L, half_y ? (float)ldexp(1.0, -ey) : 1.f, XcT + 16LL * sl * nsx * L, ldx, Bcat, ldbc, YT + 16LL * sl * L, ldg,
                                TBOA_BF16, 0, tiled | TBOA_GEMM_C_TILED | TBOA_GEMM_C_HILO | hf | (half_y ? TBOA_GEMM_C_HILO_HALF : 0));
                y.C2 = YTl + 16LL * sl * L; y.lo_scale = half_y ? 2048.f : 1.f;
                y.batch = Hkv; y.strideA = 0; y.strideB = (long long)L * ldbc; y.strideC = (long long)dm * ldg; y.tag = TBOA_PROF_AX;
                TB_TRY(gemm_bf16_nt(ctx, y));
                if (rv) {
                    y.A = XcT + 16LL * ((long long)sl * nsx + 2) * L; y.K = 4 * L; y.C = dYT + 16LL * sl * L; y.C2 = dYTl + 16LL * sl * L;
                    if (half_y) y.alpha = (float)ldexp(1.0, -ez);
                    TB_TRY(gemm_bf16_nt(ctx, y));
                }
            }
            // over the chunk: H_in^V[g] += (T1_hi + T1_lo)^T X,  R_v[g] += alpha (Z_hi + Z_lo)^T X   (X is exact, as bf16 or as half)
            const int hy = half_y ? TBOA_GEMM_F16 : 0;
            GemmBf16 h = nt(dm, dm, Gc * L, (float)ldexp(1.0, ey), YT, ldg, half_y ? XgTh : XgT, ldg, Hin_v, dm, TBOA_F32, 1, TBOA_GEMM_LOWER | tiled | hy);
            h.batch = Hkv; h.strideA = (long long)dm * ldg; h.strideB = 0; h.strideC = dd; h.tag = TBOA_PROF_HV_SYRK;
            h.flags &= ~TBOA_GEMM_PERSISTENT;
            TB_TRY(gemm_bf16_nt(ctx, h));
            h.A = YTl; if (half_y) h.alpha = (float)ldexp(1.0, ey - 11);
            TB_TRY(gemm_bf16_nt(ctx, h));
            if (rv) {
                h.tag = TBOA_PROF_RV; h.C = R_v; h.flags = tiled | hy; h.alpha = (float)ldexp(d->alpha, ez);
                h.A = dYT; TB_TRY(gemm_bf16_nt(ctx, h));
                h.A = dYTl; if (half_y) h.alpha = (float)ldexp(d->alpha, ez - 11);
                TB_TRY(gemm_bf16_nt(ctx, h));
            }
            continue;
        }
        for (int sl = 0; sl < Gc; ++sl) {
            // P = [A | A - A~];  Y^T = X_s^T A^T;  (Y - Y~)^T = [dX_s^T | X~_s^T] [A | A - A~]^T  since  A X - A~ X~ = A dX + (A - A~) X~
            if (rv) TB_TRY(scores_pair(D, Qh, Kh, Qhf, Khf, sl, Sc, Scf));
            else TB_TRY(scores(D, Qh, Kh, sl, Sc));
            TB_TRY(softmax(D, Sc, rv ? Scf : nullptr, P, ldp, -1, -1, L, bin));
            // Y^T and (Y - Y~)^T are read only by the two products below: with whole 256 x 256 tiles they are written in the
            // blocked layout of the GEMM (column offset c -> pointer offset 16 c), whose blocks those products load whole
            const long long cs = blocked ? 16 : 1;
            GemmBf16 y = nt(dm, L, L, 1.f, XcT + is * sl * nsx * L, ldx, P, ldp, YT + cs * sl * L, ldy, TBOA_BF16, 0,
                            cflag | hf | (blocked ? TBOA_GEMM_C_TILED : 0) | (bin ? TBOA_GEMM_A_TILED | TBOA_GEMM_B_TILED : 0));
            y.batch = Hq; y.batch_inner = rep; y.tag = TBOA_PROF_AX;
            y.strideB = (long long)rep * L * ldp; y.strideB2 = (long long)L * ldp;
            y.strideC = (long long)dm * ldy; y.strideC2 = cs * Gc * L;
            TB_TRY(gemm_bf16_nt(ctx, y));
            if (rv) { y.A = XcT + is * ((long long)sl * nsx + 1) * L; y.K = 2 * L; y.kseg = L; y.C = dYT + cs * sl * L; TB_TRY(gemm_bf16_nt(ctx, y)); }
        }
        const int oflag = (blocked ? (TBOA_GEMM_A_TILED | TBOA_GEMM_B_TILED) : 0) | hf;
        GemmBf16 h = nt(dm, dm, (int)ky, 1.f, YT, ldy, YT, ldy, Hin_v, dm, TBOA_F32, 1, TBOA_GEMM_LOWER | oflag);
        h.batch = Hkv; h.strideA = (long long)dm * ldy; h.strideB = h.strideA; h.strideC = dd; h.tag = TBOA_PROF_HV_SYRK;
        h.flags &= ~TBOA_GEMM_PERSISTENT;
        TB_TRY(gemm_bf16_nt(ctx, h));
        if (rv) { h.tag = TBOA_PROF_RV; h.A = dYT; h.C = R_v; h.flags = oflag; h.alpha = (float)d->alpha; TB_TRY(gemm_bf16_nt(ctx, h)); }
    }
    TB_TRY(launch_mirror_lower_f32(ctx, Hin_v, dm, Hkv));
    return 0;
}

// Operands for products with a dequantized weight W [rows, n] fp32: the integer form (hi = K, lo = NULL, *scale = step per
// row) when every row has it, else the general exact-to-16-bits pair (hi, lo), *scale = NULL; with lo2 given, three terms
// (hi, lo, lo2) that carry all 24 bits.  Synchronises once.
int weight_operands(tboa_ctx* ctx, const float* W, int rows, int n, bf16* hi, bf16* lo, float* step, const bf16** lo_out, const float** scale,
                    bf16* lo2 = nullptr, const bf16** lo2_out = nullptr) {
    int* flag = ctx->d_status + 4;
    *lo_out = lo; *scale = nullptr;
    if (lo2_out) *lo2_out = nullptr;
    TB_HIP(ctx, hipMemsetAsync(flag, 0, sizeof(int), ctx->stream));
    hipLaunchKernelGGL(int_form_kernel, dim3(rows), dim3(256), 0, ctx->stream, W, n, hi, step, flag);
    TB_KERNEL_CHECK(ctx);
    TB_HIP(ctx, hipMemcpyAsync(ctx->h_status + 4, flag, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    TB_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->h_status[4] == 0) { *lo_out = nullptr; *scale = step; ++ctx->counters[TBOA_CTR_WEIGHTS_INT_FORM]; return 0; }
    ++ctx->counters[TBOA_CTR_WEIGHTS_HILO];
    if (lo2 && lo2_out) {
        *lo2_out = lo2;
        hipLaunchKernelGGL(split_three_kernel, dim3(g1((long long)rows * n)), dim3(256), 0, ctx->stream, W, hi, lo, lo2, (long long)rows * n);
    } else
    hipLaunchKernelGGL(split_hilo_kernel, dim3(g1((long long)rows * n)), dim3(256), 0, ctx->stream, W, hi, lo, (long long)rows * n);
    TB_KERNEL_CHECK(ctx);
    return 0;
}

// (d_hi, d_lo) <- the (hi, lo) pair of (a_hi + a_lo) - (d_hi + d_lo), element by element (16-bit values: IEEE half when f16)
__global__ void pair_minus_kernel(const bf16* __restrict__ a_hi, const bf16* __restrict__ a_lo, bf16* __restrict__ d_hi, bf16* __restrict__ d_lo,
                                  long long n, int f16) {
    const long long tid = blockIdx.x * (long long)blockDim.x + threadIdx.x, nth = (long long)gridDim.x * blockDim.x;
    const long long n8 = ((((uintptr_t)a_hi | (uintptr_t)a_lo | (uintptr_t)d_hi | (uintptr_t)d_lo) & 15) == 0) ? n / 8 : 0;
    for (long long i = tid; i < n8; i += nth) {
        union { uint4 u; bf16 b[8]; } ah, al, dh, dl;
        ah.u = ((const uint4*)a_hi)[i]; al.u = ((const uint4*)a_lo)[i]; dh.u = ((const uint4*)d_hi)[i]; dl.u = ((const uint4*)d_lo)[i];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float r = (dec16(ah.b[k], f16) - dec16(dh.b[k], f16)) + (dec16(al.b[k], f16) - dec16(dl.b[k], f16));
            dh.b[k] = enc16(r, f16); dl.b[k] = enc16(r - dec16(dh.b[k], f16), f16);
        }
        ((uint4*)d_hi)[i] = dh.u; ((uint4*)d_lo)[i] = dl.u;
    }
    for (long long i = 8 * n8 + tid; i < n; i += nth) {
        const float r = (dec16(a_hi[i], f16) - dec16(d_hi[i], f16)) + (dec16(a_lo[i], f16) - dec16(d_lo[i], f16));
        const bf16 h = enc16(r, f16);
        d_hi[i] = h; d_lo[i] = enc16(r - dec16(h, f16), f16);
    }
}

// sums the (hi, lo) halves of a transposed attention output OT [dq, T (+ pad)] (IEEE half when f16) into token-major rows O [T, dq] (bf16)
__global__ __launch_bounds__(256) void ot_rows_kernel(const bf16* __restrict__ OTh, const bf16* __restrict__ OTl, long long ld, int dq,
                                                      long long T, bf16* __restrict__ O, int f16) {
    __shared__ float t[64][65];
    const long long t0 = (long long)blockIdx.x * 64; const int c0 = blockIdx.y * 64;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int c = i >> 6, tt = i & 63;
        float v = 0.f;
        if (c0 + c < dq && t0 + tt < T) {
            const long long o = (long long)(c0 + c) * ld + t0 + tt;
            v = dec16(OTh[o], f16) + dec16(OTl[o], f16);
        }
        t[c][tt] = v;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int tt = i >> 6, c = i & 63;
        if (c0 + c < dq && t0 + tt < T) O[(t0 + tt) * dq + c0 + c] = __float2bfloat16(t[c][tt]);
    }
}

// Hessian of the output projection, or (O_rows given) the attention output itself as token-major rows.
// wq_dtype: type of the weights the quantized path uses, TBOA_F32 (dequantized) or TBOA_BF16.
int build_hessian_out_proj_bf16(tboa_ctx* ctx, const tboa_attn_desc* d, const bf16* X, const bf16* X_fp, int wq_dtype, const void* Wq_deq,
                                const void* Wk_deq, const void* Wv_deq, const bf16* Wq, const bf16* Wk, const bf16* Wv, float* Hin_o,
                                float* R_o, const bf16* fp_cache, bf16* O_rows) {
    Dims D = dims_of(ctx, d);
    TB_TRY(check_bf16_dims(D));
    const int T = D.T, dm = D.dm, Hq = D.Hq, dh = D.dh, L = D.L, dq = D.dq, dkv = D.dkv, rep = D.rep;
    const bool fp = X_fp && R_o;
    int G = d->seq_chunk > 0 ? d->seq_chunk : 8; if (G > D.S) G = D.S;
    const bool fused = d->causal && qk_blocked(D) && attn_probs_t_supported(D.L, D.dh);     // no score matrices in memory
    // segments of V^T ((hi, hi, lo) per path) and of P (the same, or (hi, lo) per path from the fused kernel: its products name
    // their three operand pairs instead of reading a repeated segment)
    const int nsg = fp ? 6 : 3, nsp = fused ? (fp ? 4 : 2) : (fp ? 6 : 3), splits = pick_splits(D.S);
    const long long TP = (long long)T + PADE, ldp = (long long)nsp * L + PADE;
    bf16 *Wqh, *Wql, *Wkh, *Wkl, *Wvh, *Wvl, *Wq3, *Wk3, *Wv3, *Qh, *Kh, *Qhf, *Khf, *P, *VTc, *OT, *OTl, *dOT, *dOTl;
    float *Qf, *Kf, *VT32, *VT32f, *Sc, *Scf, *part, *steps;
    int* amx;      // [q | k | q~ | k~] x G (see QkScale)
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        Wqh = ar.get<bf16>((size_t)dq * dm); Wql = ar.get<bf16>((size_t)dq * dm);
        Wkh = ar.get<bf16>((size_t)dkv * dm); Wkl = ar.get<bf16>((size_t)dkv * dm);
        Wvh = ar.get<bf16>((size_t)dkv * dm); Wvl = ar.get<bf16>((size_t)dkv * dm);
        Wq3 = ar.get<bf16>((size_t)dq * dm); Wk3 = ar.get<bf16>((size_t)dkv * dm); Wv3 = ar.get<bf16>((size_t)dkv * dm);
        Qf = ar.get<float>((size_t)G * L * dq); Kf = ar.get<float>((size_t)G * L * dkv); VT32 = ar.get<float>((size_t)dkv * G * L);
        VT32f = fp ? ar.get<float>((size_t)dkv * G * L) : nullptr; Scf = (fp && !fused) ? ar.get<float>((size_t)Hq * L * L) : nullptr;
        Qh = ar.get<bf16>((size_t)G * L * dq * 3); Kh = ar.get<bf16>((size_t)G * L * dkv * 3);
        Qhf = fp ? ar.get<bf16>((size_t)G * L * dq * 3) : nullptr; Khf = fp ? ar.get<bf16>((size_t)G * L * dkv * 3) : nullptr;
        Sc = fused ? nullptr : ar.get<float>((size_t)Hq * L * L); P = ar.get<bf16>((size_t)Hq * L * ldp);
        VTc = ar.get<bf16>((size_t)dkv * (G * nsg * L + PADE));
        OT = ar.get<bf16>((size_t)dq * TP); OTl = ar.get<bf16>((size_t)dq * TP);
        dOT = fp ? ar.get<bf16>((size_t)dq * TP) : nullptr; dOTl = fp ? ar.get<bf16>((size_t)dq * TP) : nullptr;
        part = ar.get<float>((size_t)splits * dq * dq);
        steps = ar.get<float>((size_t)dq + 2 * dkv);
        amx = ar.get<int>((size_t)4 * G);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    hipStream_t st = ctx->stream;
    // dequantized weights in integer form (one GEMM per product) or as three bf16 terms that carry all 24 bits (three: with two
    // terms the 2^-17 they leave out reaches the scores, and A' with them, at 1e-4)
    const bf16 *Wql_u = nullptr, *Wkl_u = nullptr, *Wvl_u = nullptr, *Wq3_u = nullptr, *Wk3_u = nullptr, *Wv3_u = nullptr;
    const float *sq = nullptr, *sk = nullptr, *sv = nullptr;
    if (wq_dtype == TBOA_F32) {
        TB_TRY(weight_operands(ctx, (const float*)Wq_deq, dq, dm, Wqh, Wql, steps, &Wql_u, &sq, Wq3, &Wq3_u));
        TB_TRY(weight_operands(ctx, (const float*)Wk_deq, dkv, dm, Wkh, Wkl, steps + dq, &Wkl_u, &sk, Wk3, &Wk3_u));
        TB_TRY(weight_operands(ctx, (const float*)Wv_deq, dkv, dm, Wvh, Wvl, steps + dq + dkv, &Wvl_u, &sv, Wv3, &Wv3_u));
    } else { Wqh = (bf16*)Wq_deq; Wkh = (bf16*)Wk_deq; Wvh = (bf16*)Wv_deq; }      // bf16 weights are exact operands as they are
    // half operands when the activations fit half; a value V = W_v x beyond the range of half (|x|_max ||w||_1 > 65504) would
    // turn infinite there and surface as a non-finite Hessian, which tboa_quantize_layer rejects
    TB_TRY(fits_half(ctx, X, fp ? X_fp : nullptr, (long long)T * dm, &D.f16));
    const int hf = D.f16 ? TBOA_GEMM_F16 : 0;
    const int cflag = (d->causal ? TBOA_GEMM_CAUSAL_K : 0) | hf;
    for (int s0 = 0; s0 < D.S; s0 += G) {
        const int Gc = (D.S - s0 < G) ? D.S - s0 : G;
        const long long t0 = (long long)s0 * L, ldv = (long long)Gc * nsg * L + PADE;
        const bf16* Xc = X + t0 * dm;
        // V'^T = Wv_deq Xc^T (fp32; the row steps of the integer form are applied by vt_segments_kernel) and the
        // full-precision V~^T = Wv X~c^T
        {
            const bf16* tv[3] = {Wv3_u, Wvl_u, Wvh};       // the smallest term first
            int first = 1;
            for (const bf16* w : tv) if (w) { TB_TRY(gemm_bf16_nt(ctx, nt(dkv, Gc * L, dm, 1.f, w, dm, Xc, dm, VT32, (long long)Gc * L, TBOA_F32, first ? 0 : 1, 0))); first = 0; }
        }
        int *aq = fused ? amx : nullptr, *ak = fused ? amx + G : nullptr;
        const int *aqf = fused ? amx + 2 * G : nullptr, *akf = fused ? amx + 3 * G : nullptr;
        TB_TRY(project_qk(D, Xc, Gc * L, Wqh, Wql_u, Wkh, Wkl_u, Qf, Kf, Qh, Kh, sq, sk, aq, ak, Wq3_u, Wk3_u));
        if (fp) {
            TB_TRY(gemm_bf16_nt(ctx, nt(dkv, Gc * L, dm, 1.f, Wv, dm, X_fp + t0 * dm, dm, VT32f, (long long)Gc * L, TBOA_F32, 0, 0)));
            if (fp_cache) {     // projections of X_fp by W_Q, W_K as tboa_build_hessians left them, with the words that say how
                Qhf = (bf16*)fp_cache + t0 * dq * 3; Khf = (bf16*)fp_cache + (long long)T * dq * 3 + t0 * dkv * 3;
                const int* words = (const int*)(fp_cache + (long long)T * (dq + dkv) * 3);
                aqf = words + s0; akf = words + D.S + s0;
            } else TB_TRY(project_qk(D, X_fp + t0 * dm, Gc * L, Wq, nullptr, Wk, nullptr, Qf, Kf, Qhf, Khf, nullptr, nullptr,
                                     fused ? amx + 2 * G : nullptr, fused ? amx + 3 * G : nullptr));
        }
        hipLaunchKernelGGL(vt_segments_kernel, dim3(g1((long long)dkv * Gc * L)), dim3(256), 0, st, VT32, sv, fp ? VT32f : nullptr, VTc, dkv, Gc, L,
                           nsg, ldv, D.f16);
        TB_KERNEL_CHECK(ctx);
        for (int sl = 0; sl < Gc; ++sl) {
            // V^T segments [V'hi | V'hi | V'lo | V~hi | V~hi | V~lo], P = [A'hi | A'lo | A'hi | A~hi | A~lo | A~hi] ([A'hi | A'lo | A~hi | A~lo] fused):
            // O^T_h = [V'hi | V'hi | V'lo] [A'hi | A'lo | A'hi]^T and O~^T_h likewise from the second halves, both left as (hi, lo)
            // pairs; the deviation O - O~ is taken from the two pairs afterwards (its 22 bits then hold 1e-5 of a difference that
            // is a few percent of either: products of single half values of V' - V~, V~ and A' - A~ left 1e-4)
            if (fused) {      // scores and softmax in one kernel, nothing of the scores stored
                const long long qo = (long long)sl * Hq * L * 3 * dh, ko = (long long)sl * D.Hkv * L * 3 * dh;
                const QkScale qs{aq + sl, ak + sl, fp ? aqf + sl : nullptr, fp ? akf + sl : nullptr};
                TB_TRY(attn_probs_rows(ctx, Qh + qo, Kh + ko, fp ? Qhf + qo : nullptr, fp ? Khf + ko : nullptr, L, Hq, rep, dh, P, ldp, D.f16, qs));
            } else {
                if (fp) TB_TRY(scores_pair(D, Qh, Kh, Qhf, Khf, sl, Sc, Scf));
                else TB_TRY(scores(D, Qh, Kh, sl, Sc));
                TB_TRY(softmax(D, Sc, fp ? Scf : nullptr, P, ldp, 2 * L, L, 3 * L, 0, 1));
            }
            const long long co = t0 + (long long)sl * L;
            const float pa = (fused && D.f16) ? 1.f / ATTN_PROBS_HALF_SCALE : 1.f;       // half probabilities from the fused kernel are scaled
            // (an attention output is a convex combination of values: it fits half where they do, and then leaves as a pair of halves)
            GemmBf16 o = nt(dh, L, 3 * L, pa, VTc + (long long)sl * nsg * L, ldv, P, ldp, OT + co, TP, TBOA_BF16, 0,
                            cflag | TBOA_GEMM_C_HILO | (D.f16 ? TBOA_GEMM_C_HILO_HALF : 0));
            o.C2 = OTl + co;
            o.kseg = L; o.batch = Hq; o.batch_inner = rep; o.tag = TBOA_PROF_PV;
            o.strideA = (long long)dh * ldv; o.strideA2 = 0;
            o.strideB = (long long)rep * L * ldp; o.strideB2 = (long long)L * ldp;
            o.strideC = (long long)rep * dh * TP; o.strideC2 = (long long)dh * TP;
            if (fused) {       // (the fused kernel leaves P in 16 x 32 blocks: a column offset c is the pointer offset 16 c)
                o.flags |= TBOA_GEMM_B_TILED;
                o.nterms = 3;
                o.termA[0] = o.A; o.termA[1] = o.A; o.termA[2] = o.A + 2 * L;
                o.termB[0] = P; o.termB[1] = P + 16LL * L; o.termB[2] = P;
            }
            TB_TRY(gemm_bf16_nt(ctx, o));
            if (fp) {       // O~^T for now
                o.A = VTc + ((long long)sl * nsg + 3) * L; o.B = P + (fused ? 16LL * 2 : 3) * L; o.C = dOT + co; o.C2 = dOTl + co;
                if (fused) {
                    o.termA[0] = o.A; o.termA[1] = o.A; o.termA[2] = o.A + 2 * L;
                    o.termB[0] = o.B; o.termB[1] = o.B + 16LL * L; o.termB[2] = o.B;
                }
                TB_TRY(gemm_bf16_nt(ctx, o));
            }
        }
    }
    if (fp) {     // (dOT, dOTl) <- O^T - O~^T
        hipLaunchKernelGGL(pair_minus_kernel, dim3(g1((long long)dq * TP / 8)), dim3(256), 0, st, OT, OTl, dOT, dOTl, (long long)dq * TP, D.f16);
        TB_KERNEL_CHECK(ctx);
    }
    if (O_rows) {
        hipLaunchKernelGGL(ot_rows_kernel, dim3((unsigned)((T + 63) / 64), (dq + 63) / 64), dim3(256), 0, st, OT, OTl, TP, dq, (long long)T, O_rows, D.f16);
        TB_KERNEL_CHECK(ctx);
        if (!Hin_o) return 0;
    }
    // H_in^O = (O_hi + O_lo)^T (O_hi + O_lo), R_o = alpha (dO_hi + dO_lo)^T (O_hi + O_lo), without the lo.lo terms (half or bf16 pairs)
    const GramPair ho[3] = {{OT, OT}, {OTl, OT}, {OT, OTl}};
    TB_TRY(gram_splitk(ctx, splits, dq, 3, ho, TP, T, 1.0, 1, part, Hin_o, D.f16));
    if (fp) {
        const GramPair ro[3] = {{dOT, OT}, {dOTl, OT}, {dOT, OTl}};
        TB_TRY(gram_splitk(ctx, splits, dq, 3, ro, TP, T, d->alpha, 0, part, R_o, D.f16));
    }
    return 0;
}

// Act[t, c] = silu(G[t, c]) U[t, c], silu(g) = g / (1 + exp(-g)); gs, us (or NULL): factors per column c of G and U,
// applied first (projections through integer-form weights)
template <typename TO>
__global__ void swiglu_kernel(const float* __restrict__ G, const float* __restrict__ U, const float* __restrict__ gs, const float* __restrict__ us,
                              int dff, TO* __restrict__ out, long long n) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
        const int c = (int)(i % dff);
        const float g = gs ? G[i] * gs[c] : G[i], u = us ? U[i] * us[c] : U[i];
        out[i] = (TO)((g / (1.0f + __expf(-g))) * u);
    }
}

// layer-wise Hessian of a plain linear layer from bf16 activations: H = X^T X, R = alpha (X - X~)^T X
int build_hessian_linear_bf16(tboa_ctx* ctx, long long T, int n, double alpha, const bf16* X, const bf16* X_fp, float* H_in, float* R) {
    if (T % 8 || n % 8) return tboa_fail(ctx, TBOA_EINVAL, "build_hessian_linear: n_tokens and d_in must be multiples of 8 for bf16 inputs");
    int splits = 1;
    for (int sp = 16; sp > 1; --sp) if (T % ((long long)sp * 256) == 0) { splits = sp; break; }
    const bool fp = X_fp && R;
    const long long TP = T + PADE;
    bf16 *XT, *dXh, *dXl; float* part;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        XT = ar.get<bf16>((size_t)n * TP);
        dXh = fp ? ar.get<bf16>((size_t)n * TP) : nullptr; dXl = fp ? ar.get<bf16>((size_t)n * TP) : nullptr;
        part = ar.get<float>((size_t)splits * n * n);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    Dims D{}; D.ctx = ctx;
    TB_TRY(transpose(D, X, fp ? X_fp : nullptr, n, (int)T, n, XT, fp ? dXh : nullptr, dXl, TP));
    TB_TRY(gram_splitk(ctx, splits, n, XT, nullptr, XT, TP, (int)T, 1.0, 1, part, H_in));
    if (fp) TB_TRY(gram_splitk(ctx, splits, n, dXh, dXl, XT, TP, (int)T, alpha, 0, part, R));
    return 0;
}

// Act = silu(X Wg^T) * (X Wu^T) for bf16 activations; weights bf16, or fp32 taken as exact-to-16-bits (hi, lo) bf16 pairs
int swiglu_forward_bf16(tboa_ctx* ctx, long long T, int d, int dff, const bf16* X, int w_dtype, const void* Wg, const void* Wu, bf16* Act) {
    if (d % 8 || dff % 8) return tboa_fail(ctx, TBOA_EINVAL, "swiglu_forward: d and d_ff must be multiples of 8 for bf16 inputs");
    const bool split = (w_dtype == TBOA_F32);
    const long long chunk = 16384;
    bf16 *Wgh = nullptr, *Wgl = nullptr, *Wuh = nullptr, *Wul = nullptr; float *G, *U, *steps = nullptr;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        if (split) {
            Wgh = ar.get<bf16>((size_t)dff * d); Wgl = ar.get<bf16>((size_t)dff * d); Wuh = ar.get<bf16>((size_t)dff * d); Wul = ar.get<bf16>((size_t)dff * d);
            steps = ar.get<float>((size_t)2 * dff);
        }
        G = ar.get<float>((size_t)chunk * dff); U = ar.get<float>((size_t)chunk * dff);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    hipStream_t st = ctx->stream;
    const bf16* g_hi = (const bf16*)Wg; const bf16* u_hi = (const bf16*)Wu;
    const bf16 *g_lo = nullptr, *u_lo = nullptr; const float *gs = nullptr, *us = nullptr;
    if (split) {   // fp32 (dequantized) weights: integer form, one GEMM each, or the (hi, lo) pair, two
        TB_TRY(weight_operands(ctx, (const float*)Wg, dff, d, Wgh, Wgl, steps, &g_lo, &gs));
        TB_TRY(weight_operands(ctx, (const float*)Wu, dff, d, Wuh, Wul, steps + dff, &u_lo, &us));
        g_hi = Wgh; u_hi = Wuh;
    }
    for (long long t0 = 0; t0 < T; t0 += chunk) {
        const int rows = (int)((T - t0 < chunk) ? T - t0 : chunk);
        const bf16* Xc = X + t0 * d;
        TB_TRY(gemm_bf16_nt(ctx, nt(rows, dff, d, 1.f, Xc, d, g_hi, d, G, dff, TBOA_F32, 0, 0)));
        TB_TRY(gemm_bf16_nt(ctx, nt(rows, dff, d, 1.f, Xc, d, u_hi, d, U, dff, TBOA_F32, 0, 0)));
        if (g_lo) TB_TRY(gemm_bf16_nt(ctx, nt(rows, dff, d, 1.f, Xc, d, g_lo, d, G, dff, TBOA_F32, 1, 0)));
        if (u_lo) TB_TRY(gemm_bf16_nt(ctx, nt(rows, dff, d, 1.f, Xc, d, u_lo, d, U, dff, TBOA_F32, 1, 0)));
        hipLaunchKernelGGL(swiglu_kernel<bf16>, dim3(g1((long long)rows * dff)), dim3(256), 0, st, G, U, gs, us, dff, Act + t0 * dff,
                           (long long)rows * dff);
        TB_KERNEL_CHECK(ctx);
    }
    return 0;
}

// Y[t, c] = G[t, c] * scale[c] + Res[t, c]  (scale, Res optional)
__global__ void linear_out_kernel(const float* __restrict__ G, const float* __restrict__ scale, const bf16* __restrict__ Res, int dout,
                                  bf16* __restrict__ Y, long long n) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
        float v = scale ? G[i] * scale[(int)(i % dout)] : G[i];
        if (Res) v += __bfloat162float(Res[i]);
        Y[i] = __float2bfloat16(v);
    }
}

// Y = X W^T (+ Res) for bf16 activations; W bf16, or fp32 (dequantized: integer form or (hi, lo) pair)
int linear_forward_bf16(tboa_ctx* ctx, long long T, int din, int dout, const bf16* X, int w_dtype, const void* W, const bf16* Res, bf16* Y) {
    if (din % 8 || dout % 8) return tboa_fail(ctx, TBOA_EINVAL, "linear_forward: d_in and d_out must be multiples of 8 for bf16 inputs");
    const bool split = (w_dtype == TBOA_F32);
    const long long chunk = 16384;
    bf16 *Wh = nullptr, *Wl = nullptr; float *G, *steps = nullptr;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        if (split) { Wh = ar.get<bf16>((size_t)dout * din); Wl = ar.get<bf16>((size_t)dout * din); steps = ar.get<float>((size_t)dout); }
        G = ar.get<float>((size_t)chunk * dout);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    const bf16* w_hi = (const bf16*)W; const bf16* w_lo = nullptr; const float* sc = nullptr;
    if (split) { TB_TRY(weight_operands(ctx, (const float*)W, dout, din, Wh, Wl, steps, &w_lo, &sc)); w_hi = Wh; }
    for (long long t0 = 0; t0 < T; t0 += chunk) {
        const int rows = (int)((T - t0 < chunk) ? T - t0 : chunk);
        TB_TRY(gemm_bf16_nt(ctx, nt(rows, dout, din, 1.f, X + t0 * din, din, w_hi, din, G, dout, TBOA_F32, 0, 0)));
        if (w_lo) TB_TRY(gemm_bf16_nt(ctx, nt(rows, dout, din, 1.f, X + t0 * din, din, w_lo, din, G, dout, TBOA_F32, 1, 0)));
        hipLaunchKernelGGL(linear_out_kernel, dim3(g1((long long)rows * dout)), dim3(256), 0, ctx->stream, G, sc, Res ? Res + t0 * dout : nullptr, dout,
                           Y + t0 * dout, (long long)rows * dout);
        TB_KERNEL_CHECK(ctx);
    }
    return 0;
}

// Min-Max per-token fake quantization (weight-activation setting, Sec. 4.2): one wavefront per token.
// The level of an element is rint(v / s) + z with the quotient in fp64.  fl32(v * fl32(1/s)) is within 2^-23 (relative) of that
// quotient, so wherever it lies further than 2^-20 |t| from a half-integer both round to the same integer; only the
// elements inside that margin (and non-finite products) take the fp64 division.
// (inv_s == 0 marks a reciprocal that fp32 cannot hold as a normal number: every element then takes the division.)
__device__ __forceinline__ float act_level(float v, double s, float inv_s, float z, float maxq) {
    const float t = v * inv_s;
    float r = rintf(t);
    const bool safe = inv_s != 0.f && fabsf(t - r) < 0.5f - (fabsf(t) * 9.5367431640625e-7f + 9.5367431640625e-7f);
    if (!safe) r = (float)rint((double)v / s);
    return fminf(fmaxf(r + z, 0.f), maxq);
}

// VEC = 16 / sizeof(T) elements per lane and load; vec == 0: element-wise (any d, any alignment).  The first NCH chunks of
// 64 * VEC elements of a row stay in registers between the two passes, further ones are read again (L2 hits).
template <typename T, int NCH>
__global__ __launch_bounds__(256) void act_fakequant_kernel(const T* __restrict__ in, T* __restrict__ out, long long ntok, int d, float maxq,
                                                            int vec) {
    constexpr int VEC = 16 / (int)sizeof(T);
    typedef float f4 __attribute__((ext_vector_type(4)));
    union Pack { f4 raw; T e[VEC]; };
    const int lane = threadIdx.x & 63;
    const long long t = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= ntok) return;
    const T* x = in + t * d; T* y = out + t * d;
    float lo = 0.f, hi = 0.f;
    Pack buf[NCH];
    if (vec) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int k = (c * 64 + lane) * VEC;
            if (k < d) {
                buf[c].raw = __builtin_nontemporal_load((const f4*)(x + k));
#pragma unroll
                for (int i = 0; i < VEC; ++i) { const float v = (float)buf[c].e[i]; lo = fminf(lo, v); hi = fmaxf(hi, v); }
            }
        }
        for (int k = (NCH * 64 + lane) * VEC; k < d; k += 64 * VEC) {
            Pack pk; pk.raw = *(const f4*)(x + k);
#pragma unroll
            for (int i = 0; i < VEC; ++i) { const float v = (float)pk.e[i]; lo = fminf(lo, v); hi = fmaxf(hi, v); }
        }
    } else {
        for (int c = lane; c < d; c += 64) { const float v = (float)x[c]; lo = fminf(lo, v); hi = fmaxf(hi, v); }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { lo = fminf(lo, __shfl_xor(lo, o, 64)); hi = fmaxf(hi, __shfl_xor(hi, o, 64)); }
    if (lo == hi) { lo = -1.f; hi = 1.f; }
    // the decision (which level) is that of fp64 arithmetic on the exact input values
    const double s = ((double)hi - (double)lo) / (double)maxq;
    const double zd = rint(-(double)lo / s);
    const double rs = 1.0 / s;
    const float inv_s = (rs >= 1.17549435e-38 && rs <= 3.4e38) ? (float)rs : 0.f, z = (float)zd;
    if (vec) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int k = (c * 64 + lane) * VEC;
            if (k < d) {
                Pack o;
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    const float q = act_level((float)buf[c].e[i], s, inv_s, z, maxq);
                    o.e[i] = (T)(float)(s * ((double)q - zd));
                }
                __builtin_nontemporal_store(o.raw, (f4*)(y + k));
            }
        }
        for (int k = (NCH * 64 + lane) * VEC; k < d; k += 64 * VEC) {
            Pack pk, o; pk.raw = *(const f4*)(x + k);
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const float q = act_level((float)pk.e[i], s, inv_s, z, maxq);
                o.e[i] = (T)(float)(s * ((double)q - zd));
            }
            __builtin_nontemporal_store(o.raw, (f4*)(y + k));
        }
    } else {
        for (int c = lane; c < d; c += 64) {
            const float q = act_level((float)x[c], s, inv_s, z, maxq);
            y[c] = (T)(float)(s * ((double)q - zd));
        }
    }
}

}  // namespace

static int check_attn_desc(tboa_ctx* ctx, const tboa_attn_desc* d) {
    if (!d) return tboa_fail(ctx, TBOA_EINVAL, "null descriptor");
    if (d->d_model <= 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0 || d->n_seqs <= 0 || d->seq_len <= 0)
        return tboa_fail(ctx, TBOA_EINVAL, "attention descriptor: non-positive dimension");
    if (d->n_q_heads % d->n_kv_heads) return tboa_fail(ctx, TBOA_EINVAL, "n_q_heads=%d must be a multiple of n_kv_heads=%d", d->n_q_heads, d->n_kv_heads);
    if (d->x_dtype != TBOA_F32 && d->x_dtype != TBOA_BF16) return tboa_fail(ctx, TBOA_EINVAL, "x_dtype must be fp32 or bf16");
    if ((long long)d->n_seqs * d->seq_len > 2147483647LL) return tboa_fail(ctx, TBOA_EINVAL, "too many tokens");
    return 0;
}

extern "C" int tboa_build_hessians(tboa_ctx* ctx, const tboa_attn_desc* d, const void* X, const void* X_fp, const void* Wq,
                                   const void* Wk, const void* Wv, const void* Wo, float* Hin_qk, float* R_qk, float* Hout_q,
                                   float* Hout_k, float* Hin_v, float* R_v, float* Hout_v, void* fp_cache) {
    if (!ctx) return TBOA_EINVAL;
    TB_TRY(check_attn_desc(ctx, d));
    if (!X || !Wq || !Wk || !Wo) return tboa_fail(ctx, TBOA_EINVAL, "build_hessians: null input");
    if (!Hin_qk && !Hin_v && !Hout_v) return tboa_fail(ctx, TBOA_EINVAL, "build_hessians: no output requested");
    if ((Hin_qk != nullptr) != (Hout_q != nullptr) || (Hin_qk != nullptr) != (Hout_k != nullptr))
        return tboa_fail(ctx, TBOA_EINVAL, "build_hessians: Hin_qk, Hout_q and Hout_k are computed together: give all three or none");
    if ((R_qk && !Hin_qk) || (R_v && !Hin_v)) return tboa_fail(ctx, TBOA_EINVAL, "build_hessians: R_qk needs Hin_qk, R_v needs Hin_v");
    if ((R_qk || R_v) && !X_fp) return tboa_fail(ctx, TBOA_EINVAL, "build_hessians: R_qk / R_v need X_fp");
    if (X_fp && Hin_qk && !R_qk) return tboa_fail(ctx, TBOA_EINVAL, "build_hessians: X_fp given without R_qk");
    if (fp_cache && !R_v) return tboa_fail(ctx, TBOA_EINVAL, "build_hessians: fp_cache is filled while R_v is built: R_v missing");
    if (fp_cache && ((uintptr_t)fp_cache & 15)) return tboa_fail(ctx, TBOA_EINVAL, "build_hessians: fp_cache must be 16-byte aligned");
    if (d->x_dtype == TBOA_F32) return build_hessians_f64(ctx, d, X, X_fp, Wq, Wk, Wv, Wo, Hin_qk, R_qk, Hout_q, Hout_k, Hin_v, R_v, Hout_v);
    return build_hessians_bf16(ctx, d, (const bf16*)X, (const bf16*)X_fp, (const bf16*)Wq, (const bf16*)Wk, (const bf16*)Wo, Hin_qk, R_qk,
                               Hout_q, Hout_k, Hin_v, R_v, Hout_v, (bf16*)fp_cache);
}

extern "C" int tboa_build_hessian_out_proj(tboa_ctx* ctx, const tboa_attn_desc* d, const void* X, const void* X_fp, const float* Wq_deq,
                                           const float* Wk_deq, const float* Wv_deq, const void* Wq, const void* Wk, const void* Wv,
                                           float* Hin_o, float* R_o, const void* fp_cache) {
    if (!ctx) return TBOA_EINVAL;
    TB_TRY(check_attn_desc(ctx, d));
    if (!X || !Wq_deq || !Wk_deq || !Wv_deq || !Hin_o) return tboa_fail(ctx, TBOA_EINVAL, "build_hessian_out_proj: null argument");
    if (R_o && (!X_fp || !Wv || (!fp_cache && (!Wq || !Wk))))
        return tboa_fail(ctx, TBOA_EINVAL, "build_hessian_out_proj: R_o needs X_fp and the full-precision weights");
    if (fp_cache && ((uintptr_t)fp_cache & 15)) return tboa_fail(ctx, TBOA_EINVAL, "build_hessian_out_proj: fp_cache must be 16-byte aligned");
    if (d->x_dtype == TBOA_F32) return build_hessian_out_proj_f64(ctx, d, X, X_fp, Wq_deq, Wk_deq, Wv_deq, Wq, Wk, Wv, Hin_o, R_o);
    return build_hessian_out_proj_bf16(ctx, d, (const bf16*)X, (const bf16*)X_fp, TBOA_F32, Wq_deq, Wk_deq, Wv_deq, (const bf16*)Wq, (const bf16*)Wk,
                                       (const bf16*)Wv, Hin_o, R_o, (const bf16*)fp_cache, nullptr);
}

// The workspace the two Hessian builds of an attention block need: their own planning code, run on a host-only context that
// stops at the point where a real call would reserve the workspace (no pointer is read before that).
extern "C" size_t tboa_hessian_workspace_bytes(const tboa_attn_desc* d) {
    tboa_ctx plan{};
    plan.plan_only = 1;
    if (check_attn_desc(&plan, d) != 0) return 0;
    const void* in = (const void*)256; float* out = (float*)256;      // never dereferenced
    int rc = tboa_build_hessians(&plan, d, in, in, in, in, in, in, out, out, out, out, out, out, out, nullptr);
    if (rc != TB_PLAN_STOP) return 0;
    rc = tboa_build_hessian_out_proj(&plan, d, in, in, out, out, out, in, in, in, out, out, nullptr);
    if (rc != TB_PLAN_STOP) return 0;
    return plan.plan_bytes;
}

extern "C" int tboa_build_hout(tboa_ctx* ctx, int d_in, int n_heads, int rep, int head_dim, const float* H_in, int w_dtype, const void* W,
                               float* H_out) {
    if (!ctx) return TBOA_EINVAL;
    if (d_in <= 0 || n_heads <= 0 || rep <= 0 || head_dim <= 0 || !H_in || !W || !H_out) return tboa_fail(ctx, TBOA_EINVAL, "build_hout: bad arguments");
    if (w_dtype != TBOA_F32 && w_dtype != TBOA_BF16) return tboa_fail(ctx, TBOA_EINVAL, "build_hout: w_dtype must be fp32 or bf16");
    const long long rows = (long long)n_heads * rep * head_dim, dd = (long long)d_in * d_in, hh = (long long)head_dim * head_dim;
    double *H64, *W64, *TW, *Ho;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        H64 = ar.get<double>((size_t)dd); W64 = ar.get<double>((size_t)rows * d_in); TW = ar.get<double>((size_t)rows * d_in);
        Ho = ar.get<double>((size_t)n_heads * hh);
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    TB_TRY(launch_cvt_f32_to_f64(ctx, H_in, H64, dd));
    TB_TRY(launch_cvt_to_f64(ctx, W, w_dtype, W64, rows * d_in));
    GemmF64 a{};      // TW = W H_in
    a.M = (int)rows; a.N = d_in; a.K = d_in; a.alpha = 1.0; a.beta = 0.0; a.A = W64; a.sam = d_in; a.sak = 1; a.B = H64; a.sbk = d_in; a.sbn = 1;
    a.C = TW; a.ldc = d_in; a.batch = 1;
    TB_TRY(gemm_f64(ctx, a));
    GemmF64 b{};      // per head of the result: sum over its rep row blocks of TW_h W_h^T
    b.M = head_dim; b.N = head_dim; b.K = d_in; b.alpha = 1.0; b.sam = d_in; b.sak = 1; b.sbk = 1; b.sbn = d_in;
    b.C = Ho; b.ldc = head_dim; b.batch = n_heads; b.strideA = (long long)rep * head_dim * d_in; b.strideB = b.strideA; b.strideC = hh;
    for (int r = 0; r < rep; ++r) {
        b.A = TW + (long long)r * head_dim * d_in; b.B = W64 + (long long)r * head_dim * d_in; b.beta = r ? 1.0 : 0.0;
        TB_TRY(gemm_f64(ctx, b));
    }
    return launch_cvt_f64_to_f32(ctx, Ho, H_out, (int64_t)n_heads * hh);
}

extern "C" int tboa_build_hout_q_kv_cache(tboa_ctx* ctx, const tboa_attn_desc* d, const void* X, const void* Wk, int kv_bits, float* Hout_q) {
    if (!ctx) return TBOA_EINVAL;
    TB_TRY(check_attn_desc(ctx, d));
    if (!X || !Wk || !Hout_q) return tboa_fail(ctx, TBOA_EINVAL, "build_hout_q_kv_cache: null argument");
    if (kv_bits < 2 || kv_bits > 8) return tboa_fail(ctx, TBOA_EINVAL, "build_hout_q_kv_cache: kv_bits=%d not in 2 .. 8", kv_bits);
    const int dm = d->d_model, Hq = d->n_q_heads, Hkv = d->n_kv_heads, dh = d->head_dim, rep = Hq / Hkv, dkv = Hkv * dh;
    const long long T = (long long)d->n_seqs * d->seq_len, hh = (long long)dh * dh;
    const bool bf = d->x_dtype == TBOA_BF16;
    if (bf && (dm % 8 || dkv % 8)) return tboa_fail(ctx, TBOA_EINVAL, "build_hout_q_kv_cache: d_model and n_kv_heads*head_dim must be multiples of 8 for bf16 inputs");
    const long long chunk = T < 16384 ? T : 16384;
    float* K32 = nullptr; double *K64, *Ho, *X64 = nullptr, *W64 = nullptr;
    for (int pass = 0; pass < 2; ++pass) {
        Arena ar(pass ? ctx->ws : nullptr);
        K64 = ar.get<double>((size_t)chunk * dkv); Ho = ar.get<double>((size_t)Hkv * hh);
        if (bf) K32 = ar.get<float>((size_t)chunk * dkv);
        else { X64 = ar.get<double>((size_t)chunk * dm); W64 = ar.get<double>((size_t)dkv * dm); }
        if (!pass) TB_TRY(tboa_ws_reserve(ctx, ar.off));
    }
    const double maxq = (double)((1 << kv_bits) - 1);
    if (!bf) TB_TRY(launch_cvt_to_f64(ctx, Wk, TBOA_F32, W64, (int64_t)dkv * dm));
    for (long long t0 = 0; t0 < T; t0 += chunk) {
        const int rows = (int)((T - t0 < chunk) ? T - t0 : chunk);
        const long long qrows = (long long)rows * Hkv;
        if (bf) {       // keys of the chunk: exact products of the bf16 inputs, fp32 accumulation
            TB_TRY(gemm_bf16_nt(ctx, nt(rows, dkv, dm, 1.f, (const bf16*)X + t0 * dm, dm, (const bf16*)Wk, dm, K32, dkv, TBOA_F32, 0, 0)));
            hipLaunchKernelGGL(row_fakequant_f64_kernel<float>, dim3((unsigned)((qrows + 3) / 4)), dim3(256), 0, ctx->stream, K32, K64, qrows, dh, maxq);
        } else {
            TB_TRY(launch_cvt_to_f64(ctx, (const float*)X + t0 * dm, TBOA_F32, X64, (int64_t)rows * dm));
            GemmF64 k{};
            k.M = rows; k.N = dkv; k.K = dm; k.alpha = 1.0; k.beta = 0.0; k.A = X64; k.sam = dm; k.sak = 1; k.B = W64; k.sbk = 1; k.sbn = dm;
            k.C = K64; k.ldc = dkv; k.batch = 1;
            TB_TRY(gemm_f64(ctx, k));
            hipLaunchKernelGGL(row_fakequant_f64_kernel<double>, dim3((unsigned)((qrows + 3) / 4)), dim3(256), 0, ctx->stream, K64, K64, qrows, dh, maxq);
        }
        TB_KERNEL_CHECK(ctx);
        GemmF64 c{};    // per KV head: Ho[g] += K^_g^T K^_g over the tokens of the chunk
        c.M = dh; c.N = dh; c.K = rows; c.alpha = 1.0; c.beta = t0 ? 1.0 : 0.0; c.A = K64; c.sam = 1; c.sak = dkv; c.B = K64; c.sbk = dkv; c.sbn = 1;
        c.C = Ho; c.ldc = dh; c.batch = Hkv; c.strideA = dh; c.strideB = dh; c.strideC = hh;
        TB_TRY(gemm_f64(ctx, c));
    }
    hipLaunchKernelGGL(bcast_heads_kernel, dim3(g1(Hq * hh)), dim3(256), 0, ctx->stream, Ho, Hout_q, rep, hh, Hq * hh);
    TB_KERNEL_CHECK(ctx);
    return 0;
}

extern "C" int tboa_attention_forward(tboa_ctx* ctx, const tboa_attn_desc* d, const void* X, int w_dtype, const void* Wq, const void* Wk,
                                      const void* Wv, void* O) {
    if (!ctx) return TBOA_EINVAL;
    TB_TRY(check_attn_desc(ctx, d));
    if (!X || !Wq || !Wk || !Wv || !O) return tboa_fail(ctx, TBOA_EINVAL, "attention_forward: null argument");
    if (w_dtype != TBOA_F32 && w_dtype != d->x_dtype) return tboa_fail(ctx, TBOA_EINVAL, "attention_forward: weights must be fp32 or of the activations' type");
    if (d->x_dtype == TBOA_F32) return attention_forward_f64(ctx, d, (const float*)X, (const float*)Wq, (const float*)Wk, (const float*)Wv, (float*)O);
    return build_hessian_out_proj_bf16(ctx, d, (const bf16*)X, nullptr, w_dtype, Wq, Wk, Wv, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, (bf16*)O);
}

extern "C" int tboa_linear_forward(tboa_ctx* ctx, int64_t n_tokens, int d_in, int d_out, int x_dtype, const void* X, int w_dtype, const void* W,
                                   const void* Res, void* Y) {
    if (!ctx) return TBOA_EINVAL;
    if (n_tokens <= 0 || n_tokens > 2147483647LL || d_in <= 0 || d_out <= 0 || !X || !W || !Y) return tboa_fail(ctx, TBOA_EINVAL, "linear_forward: bad arguments");
    if (w_dtype != TBOA_F32 && w_dtype != x_dtype) return tboa_fail(ctx, TBOA_EINVAL, "linear_forward: weights must be fp32 or of the activations' type");
    if (x_dtype == TBOA_F32) return linear_forward_f64(ctx, n_tokens, d_in, d_out, (const float*)X, (const float*)W, (const float*)Res, (float*)Y);
    if (x_dtype == TBOA_BF16) return linear_forward_bf16(ctx, n_tokens, d_in, d_out, (const bf16*)X, w_dtype, W, (const bf16*)Res, (bf16*)Y);
    return tboa_fail(ctx, TBOA_EINVAL, "linear_forward: x_dtype must be fp32 or bf16");
}

extern "C" size_t tboa_fp_cache_bytes(const tboa_attn_desc* d) {
    if (!d || d->x_dtype != TBOA_BF16 || d->n_seqs <= 0 || d->seq_len <= 0 || d->head_dim <= 0) return 0;
    // the (hi, lo) operands of every token, then one word per sequence and operand that says how they are encoded (see QkScale)
    const size_t ops = (size_t)d->n_seqs * d->seq_len * (size_t)(d->n_q_heads + d->n_kv_heads) * d->head_dim * 3 * sizeof(bf16);
    return ops + (((size_t)2 * d->n_seqs * sizeof(int) + 15) & ~(size_t)15);
}

extern "C" int tboa_act_fakequant(tboa_ctx* ctx, int64_t n_tokens, int d, int bits, int dtype, const void* X_in, void* X_out) {
    if (!ctx) return TBOA_EINVAL;
    if (n_tokens < 0 || d <= 0 || bits < 2 || bits > 8 || !X_in || !X_out) return tboa_fail(ctx, TBOA_EINVAL, "act_fakequant: bad arguments");
    if (n_tokens == 0) return 0;
    const float maxq = (float)((1 << bits) - 1);
    const unsigned grid = (unsigned)((n_tokens + 3) / 4);
    const int esz = dtype == TBOA_F32 ? 4 : 2;
    // whole 16-byte pieces per lane when every row starts on a 16-byte boundary (in place is fine: a wavefront reads a piece before it writes it)
    const int vec = (((uintptr_t)X_in | (uintptr_t)X_out) & 15) == 0 && ((long long)d * esz) % 16 == 0;
    if (dtype == TBOA_F32)
        hipLaunchKernelGGL((act_fakequant_kernel<float, 8>), dim3(grid), dim3(256), 0, ctx->stream, (const float*)X_in, (float*)X_out, (long long)n_tokens, d,
                           maxq, vec);
    else if (dtype == TBOA_BF16)
        hipLaunchKernelGGL((act_fakequant_kernel<bf16, 8>), dim3(grid), dim3(256), 0, ctx->stream, (const bf16*)X_in, (bf16*)X_out, (long long)n_tokens, d,
                           maxq, vec);
    else return tboa_fail(ctx, TBOA_EINVAL, "act_fakequant: dtype must be fp32 or bf16");
    TB_KERNEL_CHECK(ctx);
    return 0;
}

extern "C" int tboa_build_hessian_linear(tboa_ctx* ctx, int64_t n_tokens, int d_in, int x_dtype, double alpha, const void* X, const void* X_fp,
                                         float* H_in, float* R) {
    if (!ctx) return TBOA_EINVAL;
    if (n_tokens <= 0 || n_tokens > 2147483647LL || d_in <= 0 || !X || !H_in) return tboa_fail(ctx, TBOA_EINVAL, "build_hessian_linear: bad arguments");
    if ((X_fp != nullptr) != (R != nullptr)) return tboa_fail(ctx, TBOA_EINVAL, "build_hessian_linear: X_fp and R go together");
    if (x_dtype == TBOA_F32) return build_hessian_linear_f64(ctx, n_tokens, d_in, alpha, (const float*)X, (const float*)X_fp, H_in, R);
    if (x_dtype == TBOA_BF16) return build_hessian_linear_bf16(ctx, n_tokens, d_in, alpha, (const bf16*)X, (const bf16*)X_fp, H_in, R);
    return tboa_fail(ctx, TBOA_EINVAL, "build_hessian_linear: x_dtype must be fp32 or bf16");
}

extern "C" int tboa_swiglu_forward(tboa_ctx* ctx, int64_t n_tokens, int d, int d_ff, int x_dtype, const void* X, int w_dtype, const void* Wg,
                                   const void* Wu, void* Act) {
    if (!ctx) return TBOA_EINVAL;
    if (n_tokens <= 0 || n_tokens > 2147483647LL || d <= 0 || d_ff <= 0 || !X || !Wg || !Wu || !Act) return tboa_fail(ctx, TBOA_EINVAL, "swiglu_forward: bad arguments");
    if (w_dtype != TBOA_F32 && w_dtype != x_dtype) return tboa_fail(ctx, TBOA_EINVAL, "swiglu_forward: weights must be fp32 or of the activations' type");
    if (x_dtype == TBOA_F32) return swiglu_forward_f64(ctx, n_tokens, d, d_ff, (const float*)X, (const float*)Wg, (const float*)Wu, (float*)Act);
    if (x_dtype == TBOA_BF16) return swiglu_forward_bf16(ctx, n_tokens, d, d_ff, (const bf16*)X, w_dtype, Wg, Wu, (bf16*)Act);
    return tboa_fail(ctx, TBOA_EINVAL, "swiglu_forward: x_dtype must be fp32 or bf16");
}
