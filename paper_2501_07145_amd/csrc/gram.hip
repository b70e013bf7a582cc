// Linear Gram of primal features, K = PhiX PhiY^T (Sec. 1: the Gram matrix of the
// low-rank feature map is the matrix of inner products of the features).
#include "rfsf_internal.h"

namespace rfsf {
namespace {

constexpr int kTile = 64;     // output tile edge
constexpr int kK = 16;        // K slab

// Generic fp32 kernel: 64x64 output tile per workgroup, 4x4 per thread, operands staged
// through LDS with scalar loads so that any leading dimension and alignment is accepted.
__global__ __launch_bounds__(256) void gram_generic(
    const float *__restrict__ A, int64_t Nx, int64_t lda, const float *__restrict__ B, int64_t Ny,
    int64_t ldb, int64_t K, float *__restrict__ C, int64_t ldc)
{
    __shared__ float As[kK][kTile + 4];
    __shared__ float Bs[kK][kTile + 4];
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int64_t i0 = (int64_t)blockIdx.y * kTile, j0 = (int64_t)blockIdx.x * kTile;
    float acc[4][4] = {};
    for (int64_t k0 = 0; k0 < K; k0 += kK) {
        for (int e = threadIdx.x; e < kTile * kK; e += 256) {
            const int r = e / kK, kk = e % kK;
            const int64_t k = k0 + kk;
            As[kk][r] = (i0 + r < Nx && k < K) ? A[(i0 + r) * lda + k] : 0.f;
            Bs[kk][r] = (j0 + r < Ny && k < K) ? B[(j0 + r) * ldb + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = As[kk][ty * 4 + u]; b[u] = Bs[kk][tx * 4 + u]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(a[u], b[v], acc[u][v]);
        }
        __syncthreads();
    }
    for (int u = 0; u < 4; ++u)
        for (int v = 0; v < 4; ++v) {
            const int64_t i = i0 + ty * 4 + u, j = j0 + tx * 4 + v;
            if (i < Nx && j < Ny) C[i * ldc + j] = acc[u][v];
        }
}

}  // namespace

hipError_t launch_gram(const float *PhiX, int64_t Nx, int64_t ldx, const float *PhiY, int64_t Ny,
                       int64_t ldy, int64_t ncols, float *K, int64_t ldk, hipStream_t stream)
{
    if (Nx == 0 || Ny == 0) return hipSuccess;
    dim3 grid((unsigned)((Ny + kTile - 1) / kTile), (unsigned)((Nx + kTile - 1) / kTile));
    hipLaunchKernelGGL(gram_generic, grid, dim3(256), 0, stream, PhiX, Nx, ldx, PhiY, Ny, ldy, ncols, K, ldk);
    return hipGetLastError();
}

}  // namespace rfsf
