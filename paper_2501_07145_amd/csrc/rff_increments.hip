// Steps 1-2 of the RFSF-TS path: per-level random Fourier features of every time point
// (Sec. 3.1, eq. (rff); W = Z / bandwidth as in the appendix class RandomFourierFeatures)
// and their increments along time (the factors nabla phi_m of Sec. 3.2, eq. (rfsf)).
#include "rfsf_internal.h"

namespace rfsf {
namespace {

// sin and cos of x to ~1e-7 absolute for |x| up to 1e5: two-term Cody-Waite reduction by
// pi/2 with fused multiply-adds, then degree-7 / degree-8 minimax polynomials on
// [-pi/4, pi/4] and a quadrant swap. The time difference cancels leading digits, so the
// fast hardware approximations are not accurate enough here.
__device__ __forceinline__ void sincos_reduced(float x, float &s, float &c)
{
    const float kf = rintf(x * 0.636619772367581343f);
    float r = fmaf(-kf, 1.57079637050628662109375f, x);
    r = fmaf(-kf, -4.37113900018624283e-8f, r);
    const float r2 = r * r;
    const float ps = fmaf(r2, fmaf(r2, -1.9515295891e-4f, 8.3321608736e-3f), -1.6666654611e-1f);
    const float S = fmaf(r * r2, ps, r);
    const float pc = fmaf(r2, fmaf(r2, 2.443315711809948e-5f, -1.388731625493765e-3f), 4.166664568298827e-2f);
    const float C = fmaf(r2 * r2, pc, fmaf(-0.5f, r2, 1.0f));
    const int q = (int)kf;
    const float ss = (q & 1) ? C : S;
    const float cc = (q & 1) ? S : C;
    // sin flips sign in quadrants 2, 3; cos in quadrants 1, 2.
    s = __uint_as_float(__float_as_uint(ss) ^ (((unsigned)q & 2u) << 30));
    c = __uint_as_float(__float_as_uint(cc) ^ ((((unsigned)q + 1u) & 2u) << 30));
}

constexpr int kRowsPerTile = 32;

// Generic vector-ALU kernel: one thread per frequency, a workgroup walks a range of
// flattened rows (n * L + t) and carries the previous row's features in registers.
__global__ __launch_bounds__(256) void rff_increments_valu(
    const float *__restrict__ X, const float *__restrict__ W, float inv_lengthscale, float scale,
    int64_t rows, int d, int M, int F, int64_t rows_per_block, float *__restrict__ dphi)
{
    extern __shared__ float xs[];                     // kRowsPerTile * d
    const int fblocks = (F + 255) / 256;
    const int m = blockIdx.y / fblocks;
    const int a = (blockIdx.y % fblocks) * 256 + threadIdx.x;
    const bool active = a < F;
    const int64_t g0 = (int64_t)blockIdx.x * rows_per_block;          // first row whose increment we own
    const int64_t g1 = min(rows - 1, g0 + rows_per_block);            // last row we need phi of
    const float *Wm = W + (int64_t)m * d * F;
    const int64_t rf = (int64_t)M * 2 * F;
    float pc = 0.f, ps = 0.f;
    for (int64_t gt = g0; gt <= g1; gt += kRowsPerTile) {
        const int nrow = (int)min((int64_t)kRowsPerTile, g1 - gt + 1);
        __syncthreads();
        for (int i = threadIdx.x; i < nrow * d; i += 256) xs[i] = X[gt * d + i];
        __syncthreads();
        if (!active) continue;
        for (int r = 0; r < nrow; ++r) {
            float acc = 0.f;
            for (int c = 0; c < d; ++c) acc = fmaf(xs[r * d + c], Wm[(int64_t)c * F + a], acc);
            float s, co;
            sincos_reduced(acc * inv_lengthscale, s, co);
            s *= scale;
            co *= scale;
            const int64_t g = gt + r;
            if (g > g0) {
                float *dst = dphi + (g - 1) * rf + (int64_t)m * 2 * F;
                dst[a] = co - pc;
                dst[F + a] = s - ps;
            }
            pc = co;
            ps = s;
        }
    }
}

}  // namespace

hipError_t launch_rff_increments(const float *X, const float *W, float inv_lengthscale,
                                 int64_t n_seq, int64_t L, int d, int M, int F, bool bf16,
                                 float *dphi, hipStream_t stream)
{
    (void)bf16;
    const int64_t rows = n_seq * L;
    if (rows < 2) return hipSuccess;
    const int64_t rows_per_block = 256;
    const int64_t nblk = (rows - 1 + rows_per_block - 1) / rows_per_block;
    const int fblocks = (F + 255) / 256;
    dim3 grid((unsigned)nblk, (unsigned)(M * fblocks));
    const float scale = 0.5f / sqrtf((float)F);    // the consumer's two-for-one FFT wants halved increments
    hipLaunchKernelGGL(rff_increments_valu, grid, dim3(256), sizeof(float) * kRowsPerTile * d, stream,
                       X, W, inv_lengthscale, scale, rows, d, M, F, rows_per_block, dphi);
    return hipGetLastError();
}

}  // namespace rfsf
