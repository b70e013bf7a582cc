// RFSF-TRP (Sec. 3.4, eqs. (trp_def), (trp), (trp_rec); appendix class TensorizedRandomProjection):
// the increments of the random Fourier features are projected per level by an independent Gaussian
// matrix Z_m [Q x 2F] (one GEMM per level on the matrix cores, the same kernel as the feature Gram)
// and combined over time by Hadamard products,
//     A_m <- A_m + A_{m-1}(before the step) (.) (Z_m delta_m[k]),  A_0 = 1,  Phi_m = A_m / sqrt(Q).
// This file holds the second stage: the recurrence over time, one thread per (sequence, component).
#include "rfsf_internal.h"

namespace rfsf {
namespace {


// P[(n*L + k)*M*Q + m*Q + q] = Z_m . (delta_m[k] / 2)  (the projection kernel writes halved increments;
// the factor 2 is restored here). Reads are coalesced over q; B time steps are loaded per batch so
// that B*M loads are in flight per thread.
template <int kMaxLevels, int B>
__global__ __launch_bounds__(256) void trp_scan_kernel(const float *__restrict__ P, int64_t L, int M, int Q,
                                                       float *__restrict__ out, int64_t ld_out, float scale)
{
    const int64_t n = blockIdx.y;
    const int q = blockIdx.x * 256 + threadIdx.x;
    float *row = out + n * ld_out;
    if (blockIdx.x == 0 && threadIdx.x == 0) row[0] = 1.0f;
    if (q >= Q) return;
    float A[kMaxLevels];
#pragma unroll
    for (int m = 0; m < kMaxLevels; ++m) A[m] = 0.f;
    const int64_t T = L - 1, MQ = (int64_t)M * Q;
    const float *p = P + n * L * MQ + q;
    int64_t k = 0;
    for (; k + B <= T; k += B) {
        float v[B][kMaxLevels];
#pragma unroll
        for (int j = 0; j < B; ++j)
#pragma unroll
            for (int m = 0; m < kMaxLevels; ++m) v[j][m] = m < M ? p[(k + j) * MQ + (int64_t)m * Q] : 0.f;
#pragma unroll
        for (int j = 0; j < B; ++j)
#pragma unroll
            for (int m = kMaxLevels - 1; m >= 0; --m)         // descending: A[m-1] is still the old value
                if (m < M) A[m] = fmaf(m ? A[m - 1] : 1.0f, 2.0f * v[j][m], A[m]);
    }
    for (; k < T; ++k)
#pragma unroll
        for (int m = kMaxLevels - 1; m >= 0; --m)
            if (m < M) A[m] = fmaf(m ? A[m - 1] : 1.0f, 2.0f * p[k * MQ + (int64_t)m * Q], A[m]);
#pragma unroll
    for (int m = 0; m < kMaxLevels; ++m)
        if (m < M) row[1 + (int64_t)m * Q + q] = A[m] * scale;
}

}  // namespace

hipError_t launch_trp_scan(const float *P, int64_t n_seq, int64_t L, int M, int Q, float *out, int64_t ld_out,
                           hipStream_t stream)
{
    if (n_seq == 0) return hipSuccess;
    dim3 grid((unsigned)((Q + 255) / 256), (unsigned)n_seq);
    const float scale = 1.0f / sqrtf((float)Q);
    if (M <= 4)
        hipLaunchKernelGGL((trp_scan_kernel<4, 16>), grid, dim3(256), 0, stream, P, L, M, Q, out, ld_out, scale);
    else if (M <= 8)
        hipLaunchKernelGGL((trp_scan_kernel<8, 8>), grid, dim3(256), 0, stream, P, L, M, Q, out, ld_out, scale);
    else
        hipLaunchKernelGGL((trp_scan_kernel<16, 4>), grid, dim3(256), 0, stream, P, L, M, Q, out, ld_out, scale);
    return hipGetLastError();
}

}  // namespace rfsf
