// Measurement hook: what this GPU delivers on the two ceilings the kernels are priced against --
// a plain streaming copy (HBM) and a loop of independent fp64 matrix instructions (matrix cores).
// Not part of the method; benchmarks print these beside the published peaks.
#include "plan.hpp"

namespace cst {

typedef double v4f64 __attribute__((ext_vector_type(4)));
typedef double v2f64 __attribute__((ext_vector_type(2)));

// dst[i] = src[i]: a workgroup moves 16 KiB, every lane four 16-byte pieces 4 KiB apart (four loads in
// flight, then four streaming stores)
__global__ void __launch_bounds__(256)
peak_copy_kernel(const v2f64 *__restrict__ src, v2f64 *__restrict__ dst, int64_t n) {
    const int64_t i0 = int64_t(blockIdx.x) * 1024 + threadIdx.x;
    v2f64 x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) x[u] = i0 + 256 * u < n ? __builtin_nontemporal_load(src + i0 + 256 * u) : v2f64{0.0, 0.0};
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (i0 + 256 * u < n) __builtin_nontemporal_store(x[u], dst + i0 + 256 * u);
}

__global__ void __launch_bounds__(256)
peak_fill_kernel(v2f64 *__restrict__ dst, int64_t n, double v) {
    const int64_t i0 = int64_t(blockIdx.x) * 1024 + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (i0 + 256 * u < n) __builtin_nontemporal_store(v2f64{v, v}, dst + i0 + 256 * u);
}

// Every wavefront runs `iters` rounds of eight independent v_mfma_f64_16x16x4f64 chains.
// sink[2], sink[3]: cycles and wall-clock ticks (100 MHz) the first wavefront spent in the loop
__global__ void __launch_bounds__(256)
peak_mfma_kernel(int iters, double seed, double *sink) {
    const long long c0 = clock64(), w0 = wall_clock64();
    v4f64 acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = v4f64{0.0, 0.0, 0.0, 0.0};
    const double a = seed + double(threadIdx.x) * 1e-9, b = seed * 0.5;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[c], 0, 0, 0);
    }
    double s = 0.0;
#pragma unroll
    for (int c = 0; c < 8; ++c) s += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
    if (s == 12345.678) sink[0] = s;      // keeps the chains alive; never true for the seeds used
    if (blockIdx.x == 0 && threadIdx.x == 0) { sink[2] = double(clock64() - c0); sink[3] = double(wall_clock64() - w0); }
}

__global__ void __launch_bounds__(64)
peak_valu_kernel(int iters, int seed, double *sink) {
    const long long c0 = clock64(), w0 = wall_clock64();
    int x = seed + int(threadIdx.x);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) x = x * 3 + u;
    }
    if (x == 0x7fffffff) sink[0] = double(x);
    if (blockIdx.x == 0 && threadIdx.x == 0) { sink[2] = double(clock64() - c0); sink[3] = double(wall_clock64() - w0); }
}

}  // namespace cst

using namespace cst;

extern "C" conststn_status conststn_measure_peak(int what, int64_t size, int repeats, conststn_stream stream,
                                                 double *result) {
    clear_error();
    if (!result || repeats < 1 || repeats > 1000 || size < 1) { set_error("bad argument"); return CONSTSTN_EINVAL; }
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    CST_HIP(hipEventCreate(&e0));
    CST_HIP(hipEventCreate(&e1));
    struct Ev { hipEvent_t a, b; ~Ev() { (void)hipEventDestroy(a); (void)hipEventDestroy(b); } } ev{e0, e1};
    int dev = 0, cus = 256;
    CST_HIP(hipGetDevice(&dev));
    CST_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    float ms = 0.f;
    if (what == CONSTSTN_PEAK_COPY) {
        if (size > (int64_t(1) << 36) || size % 16 != 0) { set_error("copy size must be a multiple of 16, at most 64 GiB"); return CONSTSTN_EINVAL; }
        DevBuf<char> src, dst;
        CST_TRY(src.alloc(size_t(size)));
        CST_TRY(dst.alloc(size_t(size)));
        const int64_t n = size / 16;
        const unsigned grid = unsigned(div_up(n, 1024));
        peak_fill_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<v2f64 *>(src.p), n, 1.0);
        peak_copy_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<const v2f64 *>(src.p), reinterpret_cast<v2f64 *>(dst.p), n);
        CST_HIP(hipEventRecord(e0, st));
        for (int r = 0; r < repeats; ++r)
            peak_copy_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<const v2f64 *>(src.p), reinterpret_cast<v2f64 *>(dst.p), n);
        CST_HIP(hipEventRecord(e1, st));
        CST_HIP(hipEventSynchronize(e1));
        CST_HIP(hipGetLastError());
        CST_HIP(hipEventElapsedTime(&ms, e0, e1));
        *result = 2.0 * double(size) * repeats / (double(ms) * 1e-3) / 1e9;          // GB/s, read + written
        return CONSTSTN_OK;
    }
    if (what == CONSTSTN_PEAK_WRITE) {
        if (size > (int64_t(1) << 36) || size % 16 != 0) { set_error("fill size must be a multiple of 16, at most 64 GiB"); return CONSTSTN_EINVAL; }
        DevBuf<char> dst;
        CST_TRY(dst.alloc(size_t(size)));
        const int64_t n = size / 16;
        const unsigned grid = unsigned(div_up(n, 1024));
        peak_fill_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<v2f64 *>(dst.p), n, 1.0);
        CST_HIP(hipEventRecord(e0, st));
        for (int r = 0; r < repeats; ++r) peak_fill_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<v2f64 *>(dst.p), n, 2.0);
        CST_HIP(hipEventRecord(e1, st));
        CST_HIP(hipEventSynchronize(e1));
        CST_HIP(hipGetLastError());
        CST_HIP(hipEventElapsedTime(&ms, e0, e1));
        *result = double(size) * repeats / (double(ms) * 1e-3) / 1e9;                // GB/s written
        return CONSTSTN_OK;
    }
    if (what == CONSTSTN_PEAK_MFMA_CLOCK || what == CONSTSTN_PEAK_VALU_CLOCK) {
        if (size > 100000000) { set_error("at most 100000000 rounds"); return CONSTSTN_EINVAL; }
        DevBuf<double> sink;
        CST_TRY(sink.alloc(4));
        int wall_khz = 100000;
        CST_HIP(hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, dev));
        for (int r = 0; r < repeats + 1; ++r) {
            if (what == CONSTSTN_PEAK_MFMA_CLOCK) peak_mfma_kernel<<<unsigned(cus) * 4, 256, 0, st>>>(int(size), 1.0, sink.p);
            else peak_valu_kernel<<<unsigned(cus), 64, 0, st>>>(int(size), 1, sink.p);
        }
        CST_HIP(hipStreamSynchronize(st));
        CST_HIP(hipGetLastError());
        double h[4] = {0, 0, 0, 0};
        CST_HIP(hipMemcpy(h, sink.p, sizeof(h), hipMemcpyDeviceToHost));
        if (h[3] <= 0.0) { set_error("the wall clock did not advance"); return CONSTSTN_EHIP; }
        *result = h[2] / h[3] * double(wall_khz) * 1e-3;                              // MHz
        return CONSTSTN_OK;
    }
    if (what == CONSTSTN_PEAK_MFMA_F64) {
        if (size > 1000000) { set_error("at most 1000000 rounds"); return CONSTSTN_EINVAL; }
        DevBuf<double> sink;
        CST_TRY(sink.alloc(4));
        const unsigned grid = unsigned(cus) * 4;          // four workgroups of four wavefronts per CU: four per SIMD
        peak_mfma_kernel<<<grid, 256, 0, st>>>(int(size), 1.0, sink.p);
        CST_HIP(hipEventRecord(e0, st));
        for (int r = 0; r < repeats; ++r) peak_mfma_kernel<<<grid, 256, 0, st>>>(int(size), 1.0, sink.p);
        CST_HIP(hipEventRecord(e1, st));
        CST_HIP(hipEventSynchronize(e1));
        CST_HIP(hipGetLastError());
        CST_HIP(hipEventElapsedTime(&ms, e0, e1));
        const double flops = double(grid) * 4.0 * double(size) * 8.0 * 2048.0 * repeats;
        *result = flops / (double(ms) * 1e-3) / 1e12;                                 // TFLOP/s
        return CONSTSTN_OK;
    }
    set_error("unknown quantity %d", what);
    return CONSTSTN_EINVAL;
}
