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


typedef float floatx16 __attribute__((ext_vector_type(16)));

// Matrix-core kernel (fp32 operands). A workgroup of four wavefronts owns 128 frequencies of
// one level and a range of flattened rows; wavefront w owns frequencies 32w..32w+31. Per tile
// of 32 rows, theta[32 rows x 32 freq] = X_tile[32 x d] * W[d x 32] is accumulated with
// v_mfma_f32_32x32x2f32 (A = rows x channels from LDS, B = channels x frequencies held in
// registers for the whole row range). In the result a lane holds one frequency (lane % 32)
// and rows 8q + 4*(lane/32) + i, q,i = 0..3, so the time difference is local except at the
// 4-row boundaries, where the two half-wavefronts exchange one value per block of rows.
template <int KSTEPS>     // ceil(d / 2) padded: channels 2*KSTEPS
__global__ __launch_bounds__(256) void rff_increments_mfma(
    const float *__restrict__ X, const float *__restrict__ W, float inv_lengthscale, float scale,
    int64_t rows, int d, int M, int F, int64_t rows_per_block, float *__restrict__ dphi)
{
    constexpr int KP = 2 * KSTEPS;              // padded channel count
    constexpr int XS = KP | 1;                  // odd LDS row stride: conflict-free A reads
    __shared__ float xs[kRowsPerTile * XS];
    const int fblocks = (F + 127) / 128;
    const int m = blockIdx.y / fblocks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int f = (blockIdx.y % fblocks) * 128 + wave * 32 + col;     // this lane's frequency
    const bool f_ok = f < F;
    const int64_t g0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t g1 = min(rows - 1, g0 + rows_per_block);             // last row whose phi we need
    const int64_t rf = (int64_t)M * 2 * F;

    // B operand: W[m][k][f] for k = 2*kk + half, zero beyond d or F
    float breg[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        const int k = 2 * kk + half;
        breg[kk] = (f_ok && k < d) ? W[((int64_t)m * d + k) * F + f] * inv_lengthscale : 0.f;
    }
    float carry_c = 0.f, carry_s = 0.f;         // row 31 of the previous tile (lower half-wavefront)
    float *out_base = dphi + (int64_t)m * 2 * F + f;

    for (int64_t gt = g0; gt <= g1; gt += kRowsPerTile) {
        const int nrow = (int)min((int64_t)kRowsPerTile, g1 - gt + 1);
        __syncthreads();
        for (int i = threadIdx.x; i < kRowsPerTile * KP; i += 256) {
            const int r = i / KP, c = i - r * KP;
            xs[r * XS + c] = (r < nrow && c < d) ? X[(gt + r) * d + c] : 0.f;
        }
        __syncthreads();
        floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xs[col * XS + 2 * kk + half], breg[kk], acc, 0, 0, 0);

        float cs[16], sn[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            sincos_reduced(acc[v], sn[v], cs[v]);
            cs[v] *= scale;
            sn[v] *= scale;
        }
        // value of the row just above each 4-row block: from the partner half-wavefront
        float up_c[4], up_s[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float pc = __shfl_xor(cs[4 * q + 3], 32);
            const float ps = __shfl_xor(sn[4 * q + 3], 32);
            // upper half needs rows 8q+3 (partner's block q); lower half needs rows 8q-1
            // (partner's block q-1, or the previous tile for q = 0)
            if (half) { up_c[q] = pc; up_s[q] = ps; }
            else if (q < 3) { up_c[q + 1] = pc; up_s[q + 1] = ps; }
            if (q == 3 && !half) { up_c[0] = carry_c; up_s[0] = carry_s; carry_c = pc; carry_s = ps; }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * half + (v & 3);
            const float prev_c = (v & 3) ? cs[v - 1] : up_c[v >> 2];
            const float prev_s = (v & 3) ? sn[v - 1] : up_s[v >> 2];
            const int64_t g = gt + r;
            if (f_ok && r < nrow && g > g0) {
                float *dst = out_base + (g - 1) * rf;
                dst[0] = cs[v] - prev_c;
                dst[F] = sn[v] - prev_s;
            }
        }
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// float -> bfloat16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t bf16_bits(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_value(uint32_t b) { return __uint_as_float(b << 16); }

// Matrix-core kernel with bf16 operands and fp32 accumulation (v_mfma_f32_32x32x16_bf16).
// W is rounded to bf16; X is split into two bf16 terms, hi = bf16(x) and lo = bf16(x - hi),
// and both are multiplied with the same W, so that the time difference of the angles does not
// inherit the 2^-9 rounding of x itself. Same tiling and epilogue as the fp32 kernel.
template <int KSTEPS>     // ceil(d / 16): channels padded to 16*KSTEPS
__global__ __launch_bounds__(256) void rff_increments_mfma_bf16(
    const float *__restrict__ X, const float *__restrict__ W, float inv_lengthscale, float scale,
    int64_t rows, int d, int M, int F, int64_t rows_per_block, float *__restrict__ dphi)
{
    constexpr int KP = 16 * KSTEPS;
    constexpr int XS = KP + 8;                  // bf16 elements per LDS row (16-byte padded)
    __shared__ __attribute__((aligned(16))) uint16_t xhi[kRowsPerTile * XS];
    __shared__ __attribute__((aligned(16))) uint16_t xlo[kRowsPerTile * XS];
    const int fblocks = (F + 127) / 128;
    const int m = blockIdx.y / fblocks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int f = (blockIdx.y % fblocks) * 128 + wave * 32 + col;
    const bool f_ok = f < F;
    const int64_t g0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t g1 = min(rows - 1, g0 + rows_per_block);
    const int64_t rf = (int64_t)M * 2 * F;

    // B operand: lane holds W[m][16*kk + 8*half + e][f], e = 0..7, as bf16
    bf16x8 breg[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const int k = 16 * kk + 8 * half + e;
            const float w0 = (f_ok && k < d) ? W[((int64_t)m * d + k) * F + f] : 0.f;
            const float w1 = (f_ok && k + 1 < d) ? W[((int64_t)m * d + k + 1) * F + f] : 0.f;
            w[e / 2] = bf16_bits(w0) | (bf16_bits(w1) << 16);
        }
        breg[kk] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    }
    float carry_c = 0.f, carry_s = 0.f;
    float *out_base = dphi + (int64_t)m * 2 * F + f;

    for (int64_t gt = g0; gt <= g1; gt += kRowsPerTile) {
        const int nrow = (int)min((int64_t)kRowsPerTile, g1 - gt + 1);
        __syncthreads();
        for (int i = threadIdx.x; i < kRowsPerTile * KP; i += 256) {
            const int r = i / KP, c = i - r * KP;
            const float x = (r < nrow && c < d) ? X[(gt + r) * d + c] : 0.f;
            const uint32_t hi = bf16_bits(x);
            xhi[r * XS + c] = (uint16_t)hi;
            xlo[r * XS + c] = (uint16_t)bf16_bits(x - bf16_value(hi));
        }
        __syncthreads();
        floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const bf16x8 ah = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&xhi[col * XS + 16 * kk + 8 * half]));
            const bf16x8 al = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&xlo[col * XS + 16 * kk + 8 * half]));
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, breg[kk], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, breg[kk], acc, 0, 0, 0);
        }
        float cs[16], sn[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            sincos_reduced(acc[v] * inv_lengthscale, sn[v], cs[v]);
            cs[v] *= scale;
            sn[v] *= scale;
        }
        float up_c[4], up_s[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float pc = __shfl_xor(cs[4 * q + 3], 32);
            const float ps = __shfl_xor(sn[4 * q + 3], 32);
            if (half) { up_c[q] = pc; up_s[q] = ps; }
            else if (q < 3) { up_c[q + 1] = pc; up_s[q + 1] = ps; }
            if (q == 3 && !half) { up_c[0] = carry_c; up_s[0] = carry_s; carry_c = pc; carry_s = ps; }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * half + (v & 3);
            const float prev_c = (v & 3) ? cs[v - 1] : up_c[v >> 2];
            const float prev_s = (v & 3) ? sn[v - 1] : up_s[v >> 2];
            const int64_t g = gt + r;
            if (f_ok && r < nrow && g > g0) {
                float *dst = out_base + (g - 1) * rf;
                dst[0] = cs[v] - prev_c;
                dst[F] = sn[v] - prev_s;
            }
        }
    }
}

}  // namespace

hipError_t launch_rff_increments(const float *X, const float *W, float inv_lengthscale,
                                 int64_t n_seq, int64_t L, int d, int M, int F, bool bf16,
                                 float *dphi, hipStream_t stream)
{
    const int64_t rows = n_seq * L;
    if (rows < 2) return hipSuccess;
    const int64_t rows_per_block = 255;     // 256 rows of phi = eight tiles; consecutive blocks share one row
    const int64_t nblk = (rows - 1 + rows_per_block - 1) / rows_per_block;
    const float scale = 0.5f / sqrtf((float)F);    // the consumer's two-for-one FFT wants halved increments
    if (bf16) {            // the caller (API layer) has checked d <= 128
        const int fb = (F + 127) / 128;
        dim3 grid((unsigned)nblk, (unsigned)(M * fb));
#define RFSF_LAUNCH_BF16(KS)                                                                                   \
    hipLaunchKernelGGL(rff_increments_mfma_bf16<KS>, grid, dim3(256), 0, stream, X, W, inv_lengthscale, scale, \
                       rows, d, M, F, rows_per_block, dphi)
        if (d <= 16) RFSF_LAUNCH_BF16(1);
        else if (d <= 32) RFSF_LAUNCH_BF16(2);
        else if (d <= 64) RFSF_LAUNCH_BF16(4);
        else RFSF_LAUNCH_BF16(8);
#undef RFSF_LAUNCH_BF16
        return hipGetLastError();
    }
    if (d <= 64) {
        const int fb = (F + 127) / 128;
        dim3 grid((unsigned)nblk, (unsigned)(M * fb));
#define RFSF_LAUNCH_MFMA(KS)                                                                              \
    hipLaunchKernelGGL(rff_increments_mfma<KS>, grid, dim3(256), 0, stream, X, W, inv_lengthscale, scale, \
                       rows, d, M, F, rows_per_block, dphi)
        if (d <= 4) RFSF_LAUNCH_MFMA(2);
        else if (d <= 8) RFSF_LAUNCH_MFMA(4);
        else if (d <= 18) RFSF_LAUNCH_MFMA(9);
        else if (d <= 32) RFSF_LAUNCH_MFMA(16);
        else RFSF_LAUNCH_MFMA(32);
#undef RFSF_LAUNCH_MFMA
        return hipGetLastError();
    }
    const int fblocks = (F + 255) / 256;
    dim3 grid((unsigned)nblk, (unsigned)(M * fblocks));
    hipLaunchKernelGGL(rff_increments_valu, grid, dim3(256), sizeof(float) * kRowsPerTile * d, stream,
                       X, W, inv_lengthscale, scale, rows, d, M, F, rows_per_block, dphi);
    return hipGetLastError();
}

}  // namespace rfsf
