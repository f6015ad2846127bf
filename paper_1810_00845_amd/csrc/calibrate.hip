// Measured peaks of the GPU a context lives on, for the roofline figures of the benchmark: issue rates of the
// instructions the modular arithmetic is made of (register-only dependency chains at full occupancy) and the
// bandwidth of a plain device-to-device copy.  Nothing here is on the hot path.
#include "hisa_internal.hpp"

#define CAL_ITERS 2048
#define CAL_CHAINS 8

// OP: 0 v_fma_f64, 1 v_mul_f64, 2 v_add_f64, 3 v_rndne_f64 (+ v_add_f64 so that the chain stays in range: two
// instructions per link), 4 64-bit integer multiply (low half; + add, and), 5 64-bit integer multiply (high half; + add, and)
template <int OP>
__global__ __launch_bounds__(256) void issue_rate_kernel(double* out, double s1, double s2) {
    double a[CAL_CHAINS];
    for (int i = 0; i < CAL_CHAINS; i++) a[i] = s1 * (threadIdx.x + i + 1);
    for (int it = 0; it < CAL_ITERS; it++) {
#pragma unroll
        for (int i = 0; i < CAL_CHAINS; i++) {
            if (OP == 0) a[i] = __builtin_fma(a[i], s1, s2);
            if (OP == 1) a[i] = a[i] * s1;
            if (OP == 2) a[i] = a[i] + s2;
            if (OP == 3) a[i] = __builtin_rint(a[i]) + 0.0;
            if (OP == 4) {
                u64 u = (u64)__double_as_longlong(a[i]);
                u = u * 0x9E3779B97F4A7C15ULL + 12345;
                a[i] = __longlong_as_double((long long)(u & 0x3FFFFFFFFFFFFFFFULL));
            }
            if (OP == 5) {
                u64 u = (u64)__double_as_longlong(a[i]);
                u = __umul64hi(u, 0x9E3779B97F4A7C15ULL) + u;
                a[i] = __longlong_as_double((long long)(u & 0x3FFFFFFFFFFFFFFFULL));
            }
        }
    }
    double s = 0;
    for (int i = 0; i < CAL_CHAINS; i++) s += a[i];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// plain streaming copy, 16 bytes per lane per access
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

template <int OP>
static int time_rate(hisa_ctx* ctx, double* sink, int blocks, double links_per_iter, double* rate) {
    hipEvent_t e0, e1;
    HIP_TRY(ctx, hipEventCreate(&e0));
    HIP_TRY(ctx, hipEventCreate(&e1));
    hipLaunchKernelGGL(issue_rate_kernel<OP>, dim3(blocks), dim3(256), 0, ctx->stream, sink, 1.0000001, 0.5);   // warm-up
    HIP_TRY(ctx, hipEventRecord(e0, ctx->stream));
    hipLaunchKernelGGL(issue_rate_kernel<OP>, dim3(blocks), dim3(256), 0, ctx->stream, sink, 1.0000001, 0.5);
    HIP_TRY(ctx, hipEventRecord(e1, ctx->stream));
    HIP_TRY(ctx, hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    HIP_TRY(ctx, hipGetLastError());
    *rate = (double)blocks * 256.0 * CAL_ITERS * CAL_CHAINS * links_per_iter / ((double)ms * 1e-3) / 1e12;
    return HISA_OK;
}

extern "C" int hisa_calibrate(hisa_ctx* ctx, hisa_calibration* out) {
    if (!ctx || !out) return HISA_ERR_ARG;
    if (t_analysis) return fail(ctx, HISA_ERR_ARG, "no kernel runs during an analysis");
    hipDeviceProp_t prop;
    int dev = 0;
    HIP_TRY(ctx, hipGetDevice(&dev));
    HIP_TRY(ctx, hipGetDeviceProperties(&prop, dev));
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const int blocks = cus * 8;   // 8 workgroups of 4 waves per compute unit: every SIMD holds 8 waves
    Temp sink(ctx, (size_t)blocks * 256 * sizeof(double));
    if (!sink.ok()) return HISA_ERR_OOM;
    *out = hisa_calibration{};
    out->compute_units = (uint32_t)cus;
    out->clock_mhz = prop.clockRate / 1000.0;
    TRY(time_rate<0>(ctx, sink.as<double>(), blocks, 1, &out->fma_f64));
    TRY(time_rate<1>(ctx, sink.as<double>(), blocks, 1, &out->mul_f64));
    TRY(time_rate<2>(ctx, sink.as<double>(), blocks, 1, &out->add_f64));
    TRY(time_rate<3>(ctx, sink.as<double>(), blocks, 2, &out->rndne_add_f64));
    TRY(time_rate<4>(ctx, sink.as<double>(), blocks, 1, &out->mul_lo_u64));
    TRY(time_rate<5>(ctx, sink.as<double>(), blocks, 1, &out->mul_hi_u64));
    // device-to-device copy of 1 GiB (read + write counted), best of three
    const size_t bytes = (size_t)1 << 30;
    Temp a(ctx, bytes), b(ctx, bytes);
    if (!a.ok() || !b.ok()) return HISA_ERR_OOM;
    HIP_TRY(ctx, hipMemsetAsync(a.u(), 1, bytes, ctx->stream));
    hipEvent_t e0, e1;
    HIP_TRY(ctx, hipEventCreate(&e0));
    HIP_TRY(ctx, hipEventCreate(&e1));
    double best = 0.0;
    for (int rep = 0; rep < 4; rep++) {
        HIP_TRY(ctx, hipEventRecord(e0, ctx->stream));
        hipLaunchKernelGGL(copy_kernel, dim3(cus * 16), dim3(256), 0, ctx->stream, (const uint4*)a.u(), (uint4*)b.u(), bytes / 16);
        HIP_TRY(ctx, hipEventRecord(e1, ctx->stream));
        HIP_TRY(ctx, hipEventSynchronize(e1));
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, e0, e1));
        const double gbs = 2.0 * (double)bytes / ((double)ms * 1e-3) / 1e9;
        if (rep > 0 && gbs > best) best = gbs;
    }
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    HIP_TRY(ctx, hipGetLastError());
    out->copy_GBs = best;
    out->copy_bytes = (uint64_t)bytes;
    return HISA_OK;
}
