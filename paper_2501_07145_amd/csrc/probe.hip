// Benchmark helper, not part of the method: what this GPU gives the simplest kernels of each kind, measured
// next to the published peaks that the roofline fractions are quoted against -- streaming reads, writes
// (plain and non-temporal stores) and a copy through a buffer much larger than the last-level cache, an
// issue loop of fp32 matrix instructions and one of fp32 fused multiply-adds.
#include "rfsf_internal.h"

namespace rfsf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_read_kernel(const floatx4 *__restrict__ src, int64_t n4, float *sink)
{
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        const floatx4 v = src[i];
        acc += v;
    }
    const float s = acc[0] + acc[1] + acc[2] + acc[3];
    if (s == 1.2345678e33f) *sink = s;           // never true for the zero-filled buffer; keeps the loads alive
}

template <bool NT>
__global__ __launch_bounds__(256) void probe_write_kernel(floatx4 *__restrict__ dst, int64_t n4)
{
    const floatx4 v = {0.f, 0.f, 0.f, 0.f};
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        if (NT) __builtin_nontemporal_store(v, dst + i);
        else dst[i] = v;
    }
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const floatx4 *__restrict__ src, floatx4 *__restrict__ dst, int64_t n4)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) dst[i] = src[i];
}

// four independent chains of v_mfma_f32_32x32x2f32 per wavefront: 4 * 4096 flop per iteration
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iterations, float *sink)
{
    floatx16 c0 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    floatx16 c1 = c0, c2 = c0, c3 = c0;
    const float a = 1.0f + 1e-3f * (float)(threadIdx.x & 7), b = 1.0f - 1e-3f * (float)(threadIdx.x & 3);
    for (int i = 0; i < iterations; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, a, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, b, c3, 0, 0, 0);
    }
    const float s = c0[0] + c1[1] + c2[2] + c3[3];
    if (s == 1.2345678e33f) *sink = s;
}

// eight independent chains of fused multiply-adds per lane: 16 flop per lane and iteration
__global__ __launch_bounds__(256) void probe_valu_kernel(int iterations, float *sink)
{
    float x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = 1e-3f * (float)(threadIdx.x + j);
    const float m = 0.999f, a = 1e-4f;
    for (int i = 0; i < iterations; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = fmaf(x[j], m, a);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += x[j];
    if (s == 1.2345678e33f) *sink = s;
}

// average milliseconds of `reps` runs of `launch` after one untimed run; negative on a HIP error
template <typename Launch>
double timed_ms(hipStream_t stream, int reps, Launch &&launch)
{
    hipEvent_t t0, t1;
    if (hipEventCreate(&t0) != hipSuccess) return -1.0;
    if (hipEventCreate(&t1) != hipSuccess) { (void)hipEventDestroy(t0); return -1.0; }
    launch();
    float ms = -1.f;
    bool ok = hipEventRecord(t0, stream) == hipSuccess;
    for (int r = 0; ok && r < reps; ++r) launch();
    ok = ok && hipEventRecord(t1, stream) == hipSuccess && hipEventSynchronize(t1) == hipSuccess &&
         hipEventElapsedTime(&ms, t0, t1) == hipSuccess && hipGetLastError() == hipSuccess;
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    return ok ? (double)ms / reps : -1.0;
}

}  // namespace

hipError_t probe_peaks(void *scratch, size_t bytes, double out[6], hipStream_t stream)
{
    const int64_t n4 = (int64_t)(bytes / 32) * 2;           // float4 elements, an even count
    if (n4 < 2) return hipErrorInvalidValue;
    floatx4 *buf = static_cast<floatx4 *>(scratch);
    float *sink = reinterpret_cast<float *>(scratch);
    hipError_t e = hipMemsetAsync(scratch, 0, bytes, stream);
    if (e != hipSuccess) return e;
    const dim3 grid(256 * 32), block(256);                     // 32 workgroups per CU's worth of grid-stride loops
    const int reps = 5;
    const double gb = (double)n4 * 16.0 / 1e9;
    const double t_read = timed_ms(stream, reps, [&] { hipLaunchKernelGGL(probe_read_kernel, grid, block, 0, stream, buf, n4, sink); });
    const double t_write = timed_ms(stream, reps, [&] { hipLaunchKernelGGL(probe_write_kernel<false>, grid, block, 0, stream, buf, n4); });
    const double t_nt = timed_ms(stream, reps, [&] { hipLaunchKernelGGL(probe_write_kernel<true>, grid, block, 0, stream, buf, n4); });
    const double t_copy = timed_ms(stream, reps, [&] { hipLaunchKernelGGL(probe_copy_kernel, grid, block, 0, stream, buf, buf + n4 / 2, n4 / 2); });
    const int iterations = 4096;
    const dim3 cgrid(256 * 4);                                 // four workgroups of four wavefronts per CU
    const double t_mfma = timed_ms(stream, reps, [&] { hipLaunchKernelGGL(probe_mfma_kernel, cgrid, block, 0, stream, iterations, sink); });
    const double t_valu = timed_ms(stream, reps, [&] { hipLaunchKernelGGL(probe_valu_kernel, dim3(256 * 8), block, 0, stream, 8 * iterations, sink); });
    if (t_read <= 0 || t_write <= 0 || t_nt <= 0 || t_copy <= 0 || t_mfma <= 0 || t_valu <= 0) return hipErrorUnknown;
    out[0] = gb / (t_read * 1e-3);
    out[1] = gb / (t_write * 1e-3);
    out[2] = gb / (t_nt * 1e-3);
    out[3] = gb / (t_copy * 1e-3);                             // bytes read plus bytes written
    out[4] = (double)cgrid.x * 4 * iterations * 4 * 4096.0 / (t_mfma * 1e-3) / 1e12;
    out[5] = (double)256 * 8 * 256 * (8.0 * iterations) * 16.0 / (t_valu * 1e-3) / 1e12;
    return hipSuccess;
}

}  // namespace rfsf
