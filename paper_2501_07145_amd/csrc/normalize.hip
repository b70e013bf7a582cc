// Level-wise normalisation of feature rows (appendix, class SignatureBase): each level block is
// divided by its own Euclidean norm and weighted by 1/sqrt(M+1); the level-0 column gets the
// weight alone.
#include "rfsf_internal.h"

namespace rfsf {
namespace {

constexpr int kCached = 32;        // values per lane held in registers (blocks up to 2048 numbers)

// One workgroup per row, one wavefront per level at a time (levels strided over the 4 wavefronts).
__global__ __launch_bounds__(256) void normalize_rows_kernel(float *__restrict__ Phi, int64_t ld, int M, int D)
{
    float *row = Phi + (int64_t)blockIdx.x * ld;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float w = 1.0f / sqrtf((float)(M + 1));
    if (threadIdx.x == 0) row[0] *= w;
    for (int m = wave; m < M; m += 4) {
        float *blk = row + 1 + (int64_t)m * D;
        if (D <= 64 * kCached) {                   // the block fits in registers: read once, write once
            float buf[kCached];
            float ss = 0.f;
#pragma unroll
            for (int i = 0; i < kCached; ++i) {
                const int j = lane + 64 * i;
                buf[i] = j < D ? blk[j] : 0.f;
                ss = fmaf(buf[i], buf[i], ss);
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
            if (ss > 0.f) {
                const float f = w / sqrtf(ss);
#pragma unroll
                for (int i = 0; i < kCached; ++i) {
                    const int j = lane + 64 * i;
                    if (j < D) blk[j] = buf[i] * f;
                }
            }
        } else {
            float ss = 0.f;
            for (int j = lane; j < D; j += 64) ss = fmaf(blk[j], blk[j], ss);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
            if (ss > 0.f) {
                const float f = w / sqrtf(ss);
                for (int j = lane; j < D; j += 64) blk[j] *= f;
            }
        }
    }
}

}  // namespace

hipError_t launch_normalize(float *Phi, int64_t N, int64_t ld, int M, int D, hipStream_t stream)
{
    if (N == 0) return hipSuccess;
    hipLaunchKernelGGL(normalize_rows_kernel, dim3((unsigned)N), dim3(256), 0, stream, Phi, ld, M, D);
    return hipGetLastError();
}

}  // namespace rfsf
