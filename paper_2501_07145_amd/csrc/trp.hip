// RFSF-TRP (Sec. 3.4, eqs. (trp_def), (trp), (trp_rec); appendix class TensorizedRandomProjection):
// the increments of the random Fourier features are projected per level by an independent Gaussian
// matrix Z_m [Q x 2F] (one GEMM per level on the matrix cores, the same kernel as the feature Gram)
// and combined over time by Hadamard products,
//     A_m <- A_m + A_{m-1}(before the step) (.) (Z_m delta_m[k]),  A_0 = 1,  Phi_m = A_m / sqrt(Q).
// This file holds the second stage: the recurrence over time, one thread per sequence and one or four
// components.
#include "rfsf_internal.h"

namespace rfsf {
namespace {


typedef float floatv4 __attribute__((ext_vector_type(4)));

template <int V> struct Vec;
template <> struct Vec<1> { typedef float type; };
template <> struct Vec<4> { typedef floatv4 type; };
__device__ __forceinline__ float lane_of(float v, int) { return v; }
__device__ __forceinline__ float lane_of(floatv4 v, int i) { return v[i]; }

// P[(n*L + k)*M*Q + m*Q + q] = Z_m . (delta_m[k] / 2)  (the projection kernel writes halved increments;
// the factor 2 is restored here). A thread owns V consecutive components of one sequence (V = 4: 16-byte
// loads; the threads of a sequence then read whole rows of P, and consecutive levels and time steps
// continue the same stream); B time steps are loaded per batch so that B*M loads are in flight per
// thread. The last, partial batch loads clamped rows and skips their updates.
template <int kMaxLevels, int B, int V>
__global__ __launch_bounds__(256) void trp_scan_kernel(const float *__restrict__ P, int64_t n_seq, int64_t L, int M,
                                                       int Q, float *__restrict__ out, int64_t ld_out, float scale)
{
    typedef typename Vec<V>::type vec;
    const int QV = (Q + V - 1) / V;
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n = g / QV;
    if (n >= n_seq) return;
    const int q = (int)(g - n * QV) * V;
    float *row = out + n * ld_out;
    if (q == 0) row[0] = 1.0f;
    float A[kMaxLevels][V];
#pragma unroll
    for (int m = 0; m < kMaxLevels; ++m)
#pragma unroll
        for (int i = 0; i < V; ++i) A[m][i] = 0.f;
    const int64_t T = L - 1, MQ = (int64_t)M * Q;
    const float *p = P + n * L * MQ + q;
    for (int64_t k = 0; k < T; k += B) {
        vec v[B][kMaxLevels];
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const int64_t kj = min(k + j, T - 1);
#pragma unroll
            for (int m = 0; m < kMaxLevels; ++m)
                v[j][m] = *reinterpret_cast<const vec *>(p + kj * MQ + (int64_t)min(m, M - 1) * Q);
        }
#pragma unroll
        for (int j = 0; j < B; ++j)
            if (k + j < T) {
#pragma unroll
                for (int m = kMaxLevels - 1; m >= 0; --m)         // descending: A[m-1] is still the old value
                    if (m < M) {
#pragma unroll
                        for (int i = 0; i < V; ++i)
                            A[m][i] = fmaf(m ? A[m - 1][i] : 1.0f, 2.0f * lane_of(v[j][m], i), A[m][i]);
                    }
            }
    }
#pragma unroll
    for (int m = 0; m < kMaxLevels; ++m)
        if (m < M) {
#pragma unroll
            for (int i = 0; i < V; ++i) row[1 + (int64_t)m * Q + q + i] = A[m][i] * scale;
        }
}

}  // namespace

hipError_t launch_trp_scan(const float *P, int64_t n_seq, int64_t L, int M, int Q, float *out, int64_t ld_out,
                           hipStream_t stream)
{
    if (n_seq == 0) return hipSuccess;
    const float scale = 1.0f / sqrtf((float)Q);
    // 16-byte loads need whole groups of four components and rows of P that start on 16 bytes
    const bool wide = Q % 4 == 0 && reinterpret_cast<uintptr_t>(P) % 16 == 0;
    const int64_t threads = n_seq * (wide ? Q / 4 : Q);
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 2147483647) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
#define RFSF_LAUNCH_TRP_SCAN(LEVELS, STEPS, WIDTH)                                                            \
    hipLaunchKernelGGL((trp_scan_kernel<LEVELS, STEPS, WIDTH>), grid, dim3(256), 0, stream, P, n_seq, L, M, Q, out,   \
                       ld_out, scale)
    // up to eight levels have kernels of their own (no loads for levels that do not exist); the batch length
    // keeps about 24 loads of 16 bytes, or 64 of 4 bytes, in flight per thread
#define RFSF_TRP_SCAN_CASE(LEVELS)                                                                            \
    case LEVELS:                                                                                              \
        if (wide) RFSF_LAUNCH_TRP_SCAN(LEVELS, (24 / LEVELS > 8 ? 8 : 24 / LEVELS), 4);                       \
        else RFSF_LAUNCH_TRP_SCAN(LEVELS, (64 / LEVELS > 16 ? 16 : 64 / LEVELS), 1);                          \
        break
    switch (M) {
        RFSF_TRP_SCAN_CASE(1);
        RFSF_TRP_SCAN_CASE(2);
        RFSF_TRP_SCAN_CASE(3);
        RFSF_TRP_SCAN_CASE(4);
        RFSF_TRP_SCAN_CASE(5);
        RFSF_TRP_SCAN_CASE(6);
        RFSF_TRP_SCAN_CASE(7);
        RFSF_TRP_SCAN_CASE(8);
    default:
        if (wide) RFSF_LAUNCH_TRP_SCAN(16, 1, 4);
        else RFSF_LAUNCH_TRP_SCAN(16, 4, 1);
    }
#undef RFSF_TRP_SCAN_CASE
#undef RFSF_LAUNCH_TRP_SCAN
    return hipGetLastError();
}

}  // namespace rfsf
