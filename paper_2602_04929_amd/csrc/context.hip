// Context, error reporting, workspace, and small elementwise kernels.
#include "internal.h"

int tboa_fail(tboa_ctx* ctx, int code, const char* fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

int tboa_ws_reserve(tboa_ctx* ctx, size_t bytes) {
    if (ctx->plan_only) { if (bytes > ctx->plan_bytes) ctx->plan_bytes = bytes; return TB_PLAN_STOP; }
    if (bytes <= ctx->ws_bytes) return 0;
    TB_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->ws) { TB_HIP(ctx, hipFree(ctx->ws)); ctx->ws = nullptr; ctx->ws_bytes = 0; }
    hipError_t e = hipMalloc(&ctx->ws, bytes);
    if (e != hipSuccess) {
        ctx->ws = nullptr;
        (void)hipGetLastError();
        return tboa_fail(ctx, TBOA_ENOMEM, "workspace of %zu bytes: %s", bytes, hipGetErrorString(e));
    }
    ctx->ws_bytes = bytes;
    return 0;
}

extern "C" int tboa_create(tboa_ctx** out, int hip_device, void* hip_stream) {
    if (!out) return TBOA_EINVAL;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || hip_device < 0 || hip_device >= n) return TBOA_EINVAL;
    if (hipSetDevice(hip_device) != hipSuccess) return TBOA_EHIP;
    if (chol_static_init(hip_device) != 0) return TBOA_EHIP;
    tboa_ctx* c = new tboa_ctx();
    c->device = hip_device;
    c->stream = (hipStream_t)hip_stream;
    c->err[0] = 0;
    c->ws = nullptr; c->ws_bytes = 0;
    c->d_status = nullptr; c->h_status = nullptr; c->prof_on = 0;
    c->aux = nullptr; c->ev_fork = nullptr; c->ev_join = nullptr;
    for (auto& v : c->counters) v = 0;
    if (hipMalloc(&c->d_status, 256 * sizeof(int)) != hipSuccess ||
        hipHostMalloc(&c->h_status, 256 * sizeof(int)) != hipSuccess) {
        if (c->d_status) (void)hipFree(c->d_status);
        delete c;
        return TBOA_ENOMEM;
    }
    if (hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) {
        tboa_destroy(c);
        return TBOA_EHIP;
    }
    *out = c;
    return 0;
}

extern "C" int tboa_reserve_workspace(tboa_ctx* ctx, size_t bytes) {
    if (!ctx) return TBOA_EINVAL;
    return tboa_ws_reserve(ctx, bytes);
}

int prof_begin(tboa_ctx* ctx, int tag, double flops, ProfRec& rec, bool& timed) {
    timed = ctx->prof_on && tag >= 0;
    if (!timed) return 0;
    TB_HIP(ctx, hipEventCreate(&rec.a)); TB_HIP(ctx, hipEventCreate(&rec.b));
    rec.tag = tag; rec.flops = flops;
    TB_HIP(ctx, hipEventRecord(rec.a, ctx->stream));
    return 0;
}

int prof_end(tboa_ctx* ctx, const ProfRec& rec, bool timed) {
    if (!timed) return 0;
    TB_HIP(ctx, hipEventRecord(rec.b, ctx->stream));
    ctx->prof.push_back(rec);
    return 0;
}

extern "C" int tboa_profile_enable(tboa_ctx* ctx, int on) {
    if (!ctx) return TBOA_EINVAL;
    ctx->prof_on = on ? 1 : 0;
    return 0;
}

extern "C" int tboa_profile_reset(tboa_ctx* ctx) {
    if (!ctx) return TBOA_EINVAL;
    TB_HIP(ctx, hipStreamSynchronize(ctx->stream));
    TB_HIP(ctx, hipStreamSynchronize(ctx->aux));
    for (auto& r : ctx->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    ctx->prof.clear();
    return 0;
}

extern "C" int tboa_profile_read(tboa_ctx* ctx, int tag, double* ms_total, int64_t* launches, double* flops_total) {
    if (!ctx) return TBOA_EINVAL;
    if (tag < 0 || tag >= TBOA_PROF_NTAGS) return tboa_fail(ctx, TBOA_EINVAL, "profile_read: unknown tag %d", tag);
    TB_HIP(ctx, hipStreamSynchronize(ctx->stream));
    TB_HIP(ctx, hipStreamSynchronize(ctx->aux));
    double ms = 0.0, fl = 0.0; int64_t n = 0;
    for (auto& r : ctx->prof) {
        if (r.tag != tag) continue;
        float t = 0.f;
        TB_HIP(ctx, hipEventElapsedTime(&t, r.a, r.b));
        ms += t; fl += r.flops; ++n;
    }
    if (ms_total) *ms_total = ms;
    if (launches) *launches = n;
    if (flops_total) *flops_total = fl;
    return 0;
}

extern "C" void tboa_destroy(tboa_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->aux) { (void)hipStreamSynchronize(ctx->aux); (void)hipStreamDestroy(ctx->aux); }
    if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
    if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
    for (auto& r : ctx->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (auto& t : ctx->tile_orders) (void)hipFree(t.dev);
    for (auto& t : ctx->tile_schedules) (void)hipFree(t.dev);
    if (ctx->ws) (void)hipFree(ctx->ws);
    if (ctx->d_status) (void)hipFree(ctx->d_status);
    if (ctx->h_status) (void)hipHostFree(ctx->h_status);
    delete ctx;
}

extern "C" int64_t tboa_counter(const tboa_ctx* ctx, int which) { return (ctx && which >= 0 && which < 6) ? ctx->counters[which] : -1; }
extern "C" const char* tboa_last_error(const tboa_ctx* ctx) { return ctx ? ctx->err : "null context"; }
extern "C" size_t tboa_workspace_bytes(const tboa_ctx* ctx) { return ctx ? ctx->ws_bytes : 0; }

// ------------------------------------------------------------------------------------------------
namespace {

template <typename T>
__global__ void fill_kernel(T* p, long long n, T v) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) p[i] = v;
}

template <typename S>
__device__ __forceinline__ double to_f64(S v);
template <> __device__ __forceinline__ double to_f64<float>(float v) { return (double)v; }
template <> __device__ __forceinline__ double to_f64<double>(double v) { return v; }
template <> __device__ __forceinline__ double to_f64<__hip_bfloat16>(__hip_bfloat16 v) { return (double)__bfloat162float(v); }

template <typename S>
__global__ void cvt_to_f64_kernel(const S* src, double* dst, long long n) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
        dst[i] = to_f64<S>(src[i]);
}

__global__ void cvt_f64_to_f32_kernel(const double* src, float* dst, long long n) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
        dst[i] = (float)src[i];
}

__global__ void strict_upper_kernel(double* a, int n) {
    double* m = a + (long long)blockIdx.z * n * n;
    const long long tot = (long long)n * n;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < tot; i += (long long)gridDim.x * blockDim.x) {
        const int r = (int)(i / n), c = (int)(i % n);
        if (c <= r) m[i] = 0.0;
    }
}

// upper triangle <- transpose of the lower one, 64 x 64 tiles through LDS (coalesced reads of the lower tile (tr, tc),
// coalesced writes of its mirror image (tc, tr)); grid.x runs over the tile pairs tr >= tc, grid.z over the matrices
__global__ __launch_bounds__(256) void mirror_lower_kernel(float* a, int n) {
    __shared__ float t[64][65];
    float* m = a + (long long)blockIdx.z * n * n;
    // tile pair number -> (tr, tc), tr >= tc
    int tr = (int)((sqrtf(8.f * (float)blockIdx.x + 1.f) - 1.f) * 0.5f);
    while ((long long)(tr + 1) * (tr + 2) / 2 <= (long long)blockIdx.x) ++tr;
    while ((long long)tr * (tr + 1) / 2 > (long long)blockIdx.x) --tr;
    const int tc = (int)(blockIdx.x - (long long)tr * (tr + 1) / 2);
    const int r0 = tr * 64, c0 = tc * 64;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int r = i >> 6, c = i & 63;
        t[r][c] = (r0 + r < n && c0 + c < n) ? m[(long long)(r0 + r) * n + c0 + c] : 0.f;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int c = i >> 6, r = i & 63;      // writes element (c0 + c, r0 + r) = transpose of (r0 + r, c0 + c)
        if (r0 + r < n && c0 + c < n && r0 + r > c0 + c) m[(long long)(c0 + c) * n + r0 + r] = t[r][c];
    }
}

__global__ void sub_kernel(const double* a, const double* b, double* o, long long n) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) o[i] = a[i] - b[i];
}

inline unsigned grid_for(long long n) {
    long long g = (n + 255) / 256;
    return (unsigned)(g < 1 ? 1 : (g > 16384 ? 16384 : g));
}

}  // namespace

int launch_fill_f64(tboa_ctx* ctx, double* p, int64_t n, double v) {
    if (n <= 0) return 0;
    hipLaunchKernelGGL(fill_kernel<double>, dim3(grid_for(n)), dim3(256), 0, ctx->stream, p, (long long)n, v);
    TB_KERNEL_CHECK(ctx); return 0;
}
int launch_fill_f32(tboa_ctx* ctx, float* p, int64_t n, float v) {
    if (n <= 0) return 0;
    hipLaunchKernelGGL(fill_kernel<float>, dim3(grid_for(n)), dim3(256), 0, ctx->stream, p, (long long)n, v);
    TB_KERNEL_CHECK(ctx); return 0;
}
int launch_cvt_to_f64(tboa_ctx* ctx, const void* src, int dtype, double* dst, int64_t n) {
    if (n <= 0) return 0;
    if (dtype == TBOA_F32)
        hipLaunchKernelGGL(cvt_to_f64_kernel<float>, dim3(grid_for(n)), dim3(256), 0, ctx->stream, (const float*)src, dst, (long long)n);
    else if (dtype == TBOA_BF16)
        hipLaunchKernelGGL(cvt_to_f64_kernel<__hip_bfloat16>, dim3(grid_for(n)), dim3(256), 0, ctx->stream, (const __hip_bfloat16*)src, dst, (long long)n);
    else if (dtype == TBOA_F64)
        hipLaunchKernelGGL(cvt_to_f64_kernel<double>, dim3(grid_for(n)), dim3(256), 0, ctx->stream, (const double*)src, dst, (long long)n);
    else return tboa_fail(ctx, TBOA_EINVAL, "unsupported dtype %d", dtype);
    TB_KERNEL_CHECK(ctx); return 0;
}
int launch_cvt_f32_to_f64(tboa_ctx* ctx, const float* src, double* dst, int64_t n) { return launch_cvt_to_f64(ctx, src, TBOA_F32, dst, n); }
int launch_cvt_f64_to_f32(tboa_ctx* ctx, const double* src, float* dst, int64_t n) {
    if (n <= 0) return 0;
    hipLaunchKernelGGL(cvt_f64_to_f32_kernel, dim3(grid_for(n)), dim3(256), 0, ctx->stream, src, dst, (long long)n);
    TB_KERNEL_CHECK(ctx); return 0;
}
int launch_strict_upper_f64(tboa_ctx* ctx, double* a, int n, int batch) {
    hipLaunchKernelGGL(strict_upper_kernel, dim3(grid_for((long long)n * n), 1, batch), dim3(256), 0, ctx->stream, a, n);
    TB_KERNEL_CHECK(ctx); return 0;
}
int launch_mirror_lower_f32(tboa_ctx* ctx, float* a, int n, int batch) {
    const long long nt = (n + 63) / 64;
    hipLaunchKernelGGL(mirror_lower_kernel, dim3((unsigned)(nt * (nt + 1) / 2), 1, batch), dim3(256), 0, ctx->stream, a, n);
    TB_KERNEL_CHECK(ctx); return 0;
}
int launch_sub_f64(tboa_ctx* ctx, const double* a, const double* b, double* out, int64_t n) {
    if (n <= 0) return 0;
    hipLaunchKernelGGL(sub_kernel, dim3(grid_for(n)), dim3(256), 0, ctx->stream, a, b, out, (long long)n);
    TB_KERNEL_CHECK(ctx); return 0;
}
