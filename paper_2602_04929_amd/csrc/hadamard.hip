// Randomised Walsh-Hadamard rotation of activation rows: y = (x * signs) H_d / sqrt(d), H_d the Sylvester-Hadamard
// matrix of order d = 2^k (the fixed, training-free transform that the weight-activation setting applies before
// quantization to spread outlier channels, App. B).
//
// Bound by HBM: a row is read once and written once.  One workgroup of d / 16 threads per row; every thread holds 16
// values in registers and runs a radix-16 butterfly on 4 index bits per round (the order in which the k bits are
// processed is free).  The first one takes bits 0..3 straight from 16 consecutive values (16-byte global loads); the later
// rounds fetch their values from LDS, 4 bits at a time upwards (the last one takes what is left); at the end a thread
// reads back 16 consecutive results and stores them as 16-byte vectors.  LDS word i sits at i + i / 16: the stride-16
// accesses of the consecutive layout and the stride-1 / stride-256 accesses of the rounds all spread over the 64 banks.
#include "internal.h"
#include <math.h>

namespace {

typedef __hip_bfloat16 bf16;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return __bfloat162float(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return __float2bfloat16(v); }

// in-register Walsh-Hadamard butterflies over the low NB bits of the index j of v[16]
template <int NB>
__device__ __forceinline__ void wht16(float (&v)[16]) {
#pragma unroll
    for (int h = 1; h < (1 << NB); h <<= 1)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (!(j & h)) { const float a = v[j], b = v[j | h]; v[j] = a + b; v[j | h] = a - b; }
}

__device__ __forceinline__ int lds_at(int i) { return i + (i >> 4); }

// element index held in slot j of thread t in a round that works on the nb bits [s, s + nb): the low nb bits of j are
// those bits, the other 4 - nb bits of j are bits [0, 4 - nb), the bits of t fill the rest in order
__device__ __forceinline__ int slot_index(int t, int j, int s, int nb) {
    const int w = 4 - nb;
    const int jl = j & ((1 << nb) - 1), jh = j >> nb;
    const int tl = t & ((1 << (s - w)) - 1), th = t >> (s - w);
    return jh | (tl << w) | (jl << s) | (th << (s + nb));
}

template <typename T>
__device__ __forceinline__ void load16(const T* __restrict__ p, float (&v)[16]);
template <>
__device__ __forceinline__ void load16<float>(const float* __restrict__ p, float (&v)[16]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) { const float4 a = ((const float4*)p)[q]; v[4 * q] = a.x; v[4 * q + 1] = a.y; v[4 * q + 2] = a.z; v[4 * q + 3] = a.w; }
}
template <>
__device__ __forceinline__ void load16<bf16>(const bf16* __restrict__ p, float (&v)[16]) {
    union { bf16 h[16]; uint4 u[2]; } in;
    in.u[0] = ((const uint4*)p)[0]; in.u[1] = ((const uint4*)p)[1];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = __bfloat162float(in.h[j]);
}

template <typename T>
__global__ void hadamard_rotate_kernel(const T* __restrict__ X, const float* __restrict__ signs, T* __restrict__ Y, int k, float scale) {
    extern __shared__ float row[];
    const int d = 1 << k, t = threadIdx.x;
    const T* x = X + (long long)blockIdx.x * d;
    T* y = Y + (long long)blockIdx.x * d;
    float v[16];
    // first butterfly round: bits [0, 4) from 16 consecutive values (16-byte loads)
    load16<T>(x + 16 * t, v);
    if (signs) {
        float sg[16];
        load16<float>(signs + 16 * t, sg);
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] *= sg[j];
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] *= scale;
    wht16<4>(v);
    if (k > 4) {
#pragma unroll
        for (int j = 0; j < 16; ++j) row[lds_at(16 * t + j)] = v[j];
        __syncthreads();
        const int part = (k - 4) & 3;          // the top `part` bits form a last, smaller round
        for (int s = 4; s < k; s += 4) {
            const int nb = (s + 4 <= k) ? 4 : part;
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] = row[lds_at(slot_index(t, j, s, nb))];
            if (nb == 4) wht16<4>(v); else if (nb == 3) wht16<3>(v); else if (nb == 2) wht16<2>(v); else wht16<1>(v);
#pragma unroll
            for (int j = 0; j < 16; ++j) row[lds_at(slot_index(t, j, s, nb))] = v[j];
            __syncthreads();
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = row[lds_at(16 * t + j)];
    }
    // thread t holds outputs 16 t .. 16 t + 15
    if (sizeof(T) == 2) {
        union { bf16 h[16]; uint4 u[2]; } o;
#pragma unroll
        for (int j = 0; j < 16; ++j) o.h[j] = from_f32<bf16>(v[j]);
        uint4* dst = (uint4*)(y + 16 * t);
        dst[0] = o.u[0]; dst[1] = o.u[1];
    } else {
        float4* dst = (float4*)(y + 16 * t);
#pragma unroll
        for (int q = 0; q < 4; ++q) dst[q] = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    }
}

}  // namespace

extern "C" int tboa_hadamard_rotate(tboa_ctx* ctx, int64_t n_tokens, int d, int dtype, const void* X_in, const float* signs, void* X_out) {
    if (!ctx) return TBOA_EINVAL;
    if (n_tokens < 0 || !X_in || !X_out) return tboa_fail(ctx, TBOA_EINVAL, "hadamard_rotate: bad arguments");
    int k = 0;
    while ((1 << k) < d) ++k;
    if (d < 16 || d > 16384 || (1 << k) != d) return tboa_fail(ctx, TBOA_EINVAL, "hadamard_rotate: d=%d must be a power of two between 16 and 16384", d);
    if (dtype != TBOA_F32 && dtype != TBOA_BF16) return tboa_fail(ctx, TBOA_EINVAL, "hadamard_rotate: dtype must be fp32 or bf16");
    if (n_tokens > 2147483647LL) return tboa_fail(ctx, TBOA_EINVAL, "hadamard_rotate: too many tokens");
    if (((uintptr_t)X_out & 15) != 0 || ((uintptr_t)X_in & 15) != 0 || ((uintptr_t)signs & 15) != 0)
        return tboa_fail(ctx, TBOA_EINVAL, "hadamard_rotate: X_in, X_out and signs must be 16-byte aligned");
    if (n_tokens == 0) return 0;
    const int nt = d / 16;
    const size_t smem = (size_t)(d + d / 16 + 16) * sizeof(float);
    const float scale = (float)(1.0 / sqrt((double)d));
    if (dtype == TBOA_F32) {
        TB_HIP(ctx, hipFuncSetAttribute((const void*)hadamard_rotate_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        hipLaunchKernelGGL(hadamard_rotate_kernel<float>, dim3((unsigned)n_tokens), dim3(nt), smem, ctx->stream, (const float*)X_in, signs, (float*)X_out, k, scale);
    } else {
        TB_HIP(ctx, hipFuncSetAttribute((const void*)hadamard_rotate_kernel<bf16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        hipLaunchKernelGGL(hadamard_rotate_kernel<bf16>, dim3((unsigned)n_tokens), dim3(nt), smem, ctx->stream, (const bf16*)X_in, signs, (bf16*)X_out, k, scale);
    }
    TB_KERNEL_CHECK(ctx);
    return 0;
}
