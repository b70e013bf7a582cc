// RFSF-DP-1D features (Sec. 3.3, eq. (dp1d)): F independent size-1 copies of the one-dimensional
// random Fourier signature feature map (static map of Sec. 3.1, eq. (rff_1d), scale of the appendix
// class RandomFourierFeatures1D; recursion of Sec. 3.2, eq. (rfsf_rec), p = 1):
//     phi_m(x)[i] = sqrt(2) cos((x . W_m[:, i]) / lengthscale + bias_m[i])
//     A_m[i] <- A_m[i] + A_{m-1}[i](before the step) * (phi_m(x_k)[i] - phi_m(x_{k-1})[i]),  A_0 = 1
//     out[n, 1 + (m-1) F + i] = A_m[i] / sqrt(F),  out[n, 0] = 1.
// One fused kernel, nothing but X, W and bias is read: components never interact, so no sketch and
// no FFT are needed and the increments never leave the chip.
#include "rfsf_internal.h"
#include "sincos.h"

namespace rfsf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
constexpr int kRows = 32;          // time points per tile

// Workgroup = (sequence, slab of 256 components), four wavefronts of 64 components each. Per tile of
// 32 time points and per level: theta = X_tile * W_m on the matrix cores (two 32x32 blocks per
// wavefront), sqrt(2) cos, transposed through a wavefront-private LDS tile so that lane c then owns
// component c for all 32 rows and runs the recurrence down the rows. E[r] carries, from one level
// to the next, the value of the previous level's accumulator before row r.
template <int KSTEPS>
__global__ __launch_bounds__(256) void dp1d_features_kernel(
    const float *__restrict__ X, const float *__restrict__ W, const float *__restrict__ bias,
    float inv_lengthscale, int64_t L, int d, int M, int F, float *__restrict__ out, int64_t ld_out)
{
    constexpr int KP = 2 * KSTEPS, XS = KP | 1;
    __shared__ float xs[2 * kRows * XS];
    __shared__ float tile[4][kRows][65];
    extern __shared__ float level_state[];             // [2][M][256]: accumulators, then last cosines
    float (*acc_state)[256] = reinterpret_cast<float (*)[256]>(level_state);
    float (*cos_state)[256] = reinterpret_cast<float (*)[256]>(level_state + (size_t)M * 256);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int64_t n = blockIdx.x;
    const int comp0 = blockIdx.y * 256 + wave * 64;
    const int my_comp = comp0 + lane;
    const float *xseq = X + n * L * d;
    for (int m = 0; m < M; ++m) acc_state[m][tid] = 0.f;

    constexpr int NX = (kRows * KP + 255) / 256;
    float xr[NX];
    auto fetch_tile = [&](int64_t t0) {
        const int nrow = (int)min((int64_t)kRows, L - t0);
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            const int i = tid + 256 * u;
            const int r = i / KP, c = i - r * KP;
            xr[u] = (i < kRows * KP && r < nrow && c < d) ? xseq[(t0 + r) * d + c] : 0.f;
        }
    };
    auto put_tile = [&](float *buf) {
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            const int i = tid + 256 * u;
            const int r = i / KP, c = i - r * KP;
            if (i < kRows * KP) buf[r * XS + c] = xr[u];
        }
    };
    fetch_tile(0);
    put_tile(xs);
    __syncthreads();
    int cur = 0;
    for (int64_t t0 = 0; t0 < L; t0 += kRows, cur ^= 1) {
        const int nrow = (int)min((int64_t)kRows, L - t0);
        const bool more = t0 + kRows < L;
        if (more) fetch_tile(t0 + kRows);
        const float *xt = xs + cur * (kRows * XS);
        float E[kRows];
        for (int m = 0; m < M; ++m) {
            // projection, bias, cosine: two blocks of 32 components
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const int f = comp0 + cb * 32 + col;
                const bool f_ok = f < F;
                floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KSTEPS; ++kk) {
                    const int k = 2 * kk + half;
                    const float b = (f_ok && k < d) ? W[((int64_t)m * d + k) * F + f] * inv_lengthscale : 0.f;
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xt[col * XS + k], b, acc, 0, 0, 0);
                }
                const float bm = f_ok ? bias[(int64_t)m * F + f] : 0.f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float s, c;
                    sincos_reduced(acc[v] + bm, s, c);
                    tile[wave][8 * (v >> 2) + 4 * half + (v & 3)][cb * 32 + col] = 1.41421356237309505f * c;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // recurrence down the rows for this lane's component
            float a = acc_state[m][tid];
            float pc = t0 == 0 ? tile[wave][0][lane] : cos_state[m][tid];   // first point: no increment
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                const float c = tile[wave][r][lane];
                const float u = r < nrow ? c - pc : 0.f;
                pc = r < nrow ? c : pc;
                const float e_old = m == 0 ? 1.0f : E[r];
                E[r] = a;
                a = fmaf(e_old, u, a);
            }
            acc_state[m][tid] = a;
            cos_state[m][tid] = pc;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        if (more) put_tile(xs + (cur ^ 1) * (kRows * XS));
        __syncthreads();
    }
    float *row = out + n * ld_out;
    if (blockIdx.y == 0 && tid == 0) row[0] = 1.0f;
    const float scale = 1.0f / sqrtf((float)F);
    if (my_comp < F)
        for (int m = 0; m < M; ++m) row[1 + (int64_t)m * F + my_comp] = acc_state[m][tid] * scale;
}

}  // namespace

hipError_t launch_dp1d(const float *X, const float *W, const float *bias, float inv_lengthscale, int64_t N,
                       int64_t L, int d, int M, int F, float *out, int64_t ld_out, hipStream_t stream)
{
    if (N == 0) return hipSuccess;
    dim3 grid((unsigned)N, (unsigned)((F + 255) / 256));
    const size_t dyn = sizeof(float) * 2 * (size_t)M * 256;
    // static LDS of the kernel (X double buffer + transposition tiles) plus the per-level state can pass
    // 64 KB for many levels on a wide state; the limit on the dynamic part is then raised once per kernel
#define RFSF_LAUNCH_DP1D(KS)                                                                                  \
    do {                                                                                                      \
        constexpr size_t kStatic = sizeof(float) * (2 * kRows * ((2 * KS) | 1) + 4 * kRows * 65);             \
        static size_t raised = 0;                                                                             \
        if (kStatic + dyn > 64 * 1024 && dyn > raised) {                                                      \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(dp1d_features_kernel<KS>),      \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);         \
            if (e != hipSuccess) return e;                                                                    \
            raised = dyn;                                                                                     \
        }                                                                                                     \
        hipLaunchKernelGGL(dp1d_features_kernel<KS>, grid, dim3(256), dyn, stream, X, W, bias,                \
                           inv_lengthscale, L, d, M, F, out, ld_out);                                         \
    } while (0)
    if (d <= 4) RFSF_LAUNCH_DP1D(2);
    else if (d <= 8) RFSF_LAUNCH_DP1D(4);
    else if (d <= 18) RFSF_LAUNCH_DP1D(9);
    else if (d <= 32) RFSF_LAUNCH_DP1D(16);
    else RFSF_LAUNCH_DP1D(32);
#undef RFSF_LAUNCH_DP1D
    return hipGetLastError();
}

}  // namespace rfsf
