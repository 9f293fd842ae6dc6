// Deployable form of a quantized weight: the b-bit codes of a row packed into a little-endian bit stream
// (code c occupies bits [b c, b c + b) of the row's stream, the stream is stored as 32-bit words and a row is padded to
// whole words), and a check that the packed form carries the layer: y = W_deq x computed from the packed codes, the
// scales and the zero points alone.  The memory footprint of the weights is what weight quantization is for (Sec. 1).
#include "internal.h"

namespace {

// one thread per output word: gathers the codes whose bits fall into the word (a 3-bit code may straddle two words)
__global__ void pack_codes_kernel(const uint8_t* __restrict__ codes, int d_out, int d_in, int bits, int wpr, uint32_t* __restrict__ packed) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long long)d_out * wpr) return;
    const int r = (int)(i / wpr), w = (int)(i % wpr);
    const uint8_t* row = codes + (long long)r * d_in;
    const long long b0 = 32LL * w;                      // first bit of the word in the row's stream
    const int c0 = (int)(b0 / bits);
    int c1 = (int)((b0 + 31) / bits); if (c1 >= d_in) c1 = d_in - 1;
    uint32_t out = 0;
    for (int c = c0; c <= c1; ++c) {
        const long long pos = (long long)c * bits - b0;  // may be negative: the code started in the previous word
        const uint32_t v = row[c];
        out |= (pos >= 0) ? (v << pos) : (v >> (-pos));
    }
    packed[i] = out;
}

__device__ __forceinline__ uint32_t code_at(const uint32_t* __restrict__ words, int c, int bits, int wpr) {
    const long long pos = (long long)c * bits;
    const int w = (int)(pos >> 5), sh = (int)(pos & 31);
    uint32_t v = words[w] >> sh;
    if (sh + bits > 32 && w + 1 < wpr) v |= words[w + 1] << (32 - sh);
    return v & ((1u << bits) - 1u);
}

// one wavefront per row: y[r] = sum_c scales[r, c / g] (code[r, c] - zeros[r, c / g]) x[c]
__global__ __launch_bounds__(256) void dequant_gemv_kernel(const uint32_t* __restrict__ packed, const float* __restrict__ scales,
                                                           const float* __restrict__ zeros, const float* __restrict__ x, int d_out, int d_in,
                                                           int bits, int gsz, int ng, int wpr, float* __restrict__ y) {
    const int lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= d_out) return;
    const uint32_t* words = packed + (long long)r * wpr;
    double acc = 0.0;
    for (int c = lane; c < d_in; c += 64) {
        const int g = c / gsz;
        const double q = (double)code_at(words, c, bits, wpr) - (double)zeros[(long long)r * ng + g];
        acc += (double)scales[(long long)r * ng + g] * q * (double)x[c];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) y[r] = (float)acc;
}

int check_pack_args(tboa_ctx* ctx, int d_out, int d_in, int bits) {
    if (d_out <= 0 || d_in <= 0) return tboa_fail(ctx, TBOA_EINVAL, "pack: d_out and d_in must be positive");
    if (!(bits == 2 || bits == 3 || bits == 4 || bits == 8)) return tboa_fail(ctx, TBOA_EINVAL, "pack: bits=%d not in {2,3,4,8}", bits);
    return 0;
}

}  // namespace

extern "C" int64_t tboa_packed_words_per_row(int d_in, int bits) {
    if (d_in <= 0 || bits <= 0) return 0;
    return ((int64_t)d_in * bits + 31) / 32;
}

extern "C" int tboa_pack_codes(tboa_ctx* ctx, int d_out, int d_in, int bits, const uint8_t* codes, uint32_t* packed) {
    if (!ctx) return TBOA_EINVAL;
    TB_TRY(check_pack_args(ctx, d_out, d_in, bits));
    if (!codes || !packed) return tboa_fail(ctx, TBOA_EINVAL, "pack_codes: null argument");
    const int wpr = (int)tboa_packed_words_per_row(d_in, bits);
    const long long n = (long long)d_out * wpr;
    hipLaunchKernelGGL(pack_codes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, codes, d_out, d_in, bits, wpr, packed);
    TB_KERNEL_CHECK(ctx);
    return 0;
}

extern "C" int tboa_dequant_gemv(tboa_ctx* ctx, int d_out, int d_in, int bits, int group, const uint32_t* packed, const float* scales,
                                 const float* zeros, const float* x, float* y) {
    if (!ctx) return TBOA_EINVAL;
    TB_TRY(check_pack_args(ctx, d_out, d_in, bits));
    if (!packed || !scales || !zeros || !x || !y) return tboa_fail(ctx, TBOA_EINVAL, "dequant_gemv: null argument");
    if (group < 0 || (group > 0 && d_in % group != 0)) return tboa_fail(ctx, TBOA_EINVAL, "dequant_gemv: group=%d must divide d_in=%d", group, d_in);
    const int gsz = group ? group : d_in, ng = d_in / gsz;
    const int wpr = (int)tboa_packed_words_per_row(d_in, bits);
    hipLaunchKernelGGL(dequant_gemv_kernel, dim3((d_out + 3) / 4), dim3(256), 0, ctx->stream, packed, scales, zeros, x, d_out, d_in, bits, gsz, ng,
                       wpr, y);
    TB_KERNEL_CHECK(ctx);
    return 0;
}
