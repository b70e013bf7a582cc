// RFSF-DP-1D features (Sec. 3.3, eq. (dp1d)): F independent size-1 copies of the one-dimensional
// random Fourier signature feature map (static map of Sec. 3.1, eq. (rff_1d), scale of the appendix
// class RandomFourierFeatures1D; recursion of Sec. 3.2, eq. (rfsf_rec), p = 1):
//     phi_m(x)[i] = sqrt(2) cos((x . W_m[:, i]) / lengthscale + bias_m[i])
//     A_m[i] <- A_m[i] + A_{m-1}[i](before the step) * (phi_m(x_k)[i] - phi_m(x_{k-1})[i]),  A_0 = 1
//     out[n, 1 + (m-1) F + i] = A_m[i] / sqrt(F),  out[n, 0] = 1.
// One fused kernel, nothing but X, W and bias is read: components never interact, so no sketch and
// no FFT are needed and the increments never leave the chip.
#include "rfsf_internal.h"

namespace rfsf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kRows = 32;          // time points per tile
constexpr int kRawBufferWord3 = 0x00020000;   // buffer descriptor, last word: untyped 32-bit data
constexpr int kTileStride = 36;    // floats per component in the transposition tile: 16-byte accesses of 16
                                   // consecutive components then fall on 16 distinct groups of four banks

// sqrt(2) cos(x) to 2.4e-7 absolute for |x| < 1e6: x = k pi + r with |r| <= pi/2 (k from adding 1.5 * 2^23,
// whose lowest mantissa bit is then the parity of k; two-term Cody-Waite reduction), a degree-5 polynomial
// in r^2 (Chebyshev interpolant of sqrt(2) cos(sqrt(u)) on [0, (pi/2)^2], 2e-10) and the sign (-1)^k.
__device__ __forceinline__ float sqrt2_cos(float x)
{
    const float t = fmaf(x, 0.318309886183790672f, 12582912.0f);
    const float kf = t - 12582912.0f;
    float r = fmaf(-kf, 3.14159274101257324f, x);
    r = fmaf(-kf, -8.74227800037248566e-8f, r);
    const float u = r * r;
    float p = fmaf(u, -3.684157832e-07f, 3.501610627e-05f);
    p = fmaf(u, p, -1.964110881e-03f);
    p = fmaf(u, p, 5.892552063e-02f);
    p = fmaf(u, p, -7.071067691e-01f);
    p = fmaf(u, p, 1.414213538e+00f);
    return __uint_as_float(__float_as_uint(p) ^ (__float_as_uint(t) << 31));
}

// orders the LDS accesses of one wavefront (the hardware runs them in program order; this keeps the
// compiler from moving them) without waiting for the global loads in flight
__device__ __forceinline__ void lds_order()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    asm volatile("" ::: "memory");
}

// The recurrence of one level down the rows of a tile for this lane's component. c: the component's
// sqrt(2) cos values in the transposition tile; E[r] holds, on entry, the previous level's accumulator
// before row r and, on exit, this level's.
template <bool FIRST_LEVEL, bool FULL>
__device__ __forceinline__ void run_rows(const float *c, bool first_tile, float (&E)[kRows], float &a, float &pc, int nrow)
{
#pragma unroll
    for (int g = 0; g < kRows / 4; ++g) {
        const floatx4 v = *reinterpret_cast<const floatx4 *>(c + 4 * g);
        if (g == 0) pc = first_tile ? v[0] : pc;           // first point of the sequence: no increment
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = 4 * g + j;
            float u = v[j] - pc;
            if (FULL) {
                pc = v[j];
            } else {
                u = r < nrow ? u : 0.f;
                pc = r < nrow ? v[j] : pc;
            }
            const float e_old = FIRST_LEVEL ? 1.0f : E[r];
            E[r] = a;
            a = fmaf(e_old, u, a);
        }
    }
}

// Workgroup = (sequence, slab of 256 components), four wavefronts of 64 components each. Per tile of
// 32 time points and per level: theta = X_tile * W_m on the matrix cores (two 32x32 blocks per
// wavefront), sqrt(2) cos, transposed through a wavefront-private LDS tile so that lane c then owns
// component c for all 32 rows and runs the recurrence down the rows. E[r] carries, from one level
// to the next, the value of the previous level's accumulator before row r. The W columns of the next
// level are fetched right after the matrix instructions of the current one and land under its cosines.
template <int KSTEPS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(KSTEPS <= 4 ? 4 : KSTEPS <= 16 ? 3 : 2, 4)))
void dp1d_features_kernel(
    const float *__restrict__ X, const float *__restrict__ W, const float *__restrict__ bias,
    float inv_lengthscale, int64_t L, int d, int M, int F, float *__restrict__ out, int64_t ld_out)
{
    constexpr int KP = 2 * KSTEPS, XS = KP | 1;
    constexpr bool kKeepX = KSTEPS <= 16;              // the tile's A fragments stay in registers for all levels
    __shared__ float xs[2 * kRows * XS];
    __shared__ __attribute__((aligned(16))) float tile[4][64 * kTileStride];
    extern __shared__ float level_state[];             // [2][M][256]: accumulators, then last cosines
    float (*acc_state)[256] = reinterpret_cast<float (*)[256]>(level_state);
    float (*cos_state)[256] = reinterpret_cast<float (*)[256]>(level_state + (size_t)M * 256);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int64_t n = blockIdx.x;
    const int comp0 = blockIdx.y * 256 + wave * 64;
    const int my_comp = comp0 + lane;
    const float *xseq = X + n * L * d;
    for (int m = 0; m < M; ++m) acc_state[m][tid] = 0.f, cos_state[m][tid] = 0.f;

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
    // B fragments: this lane's W entries of one level for its two blocks of 32 components, fetched with
    // buffer loads: one descriptor per pair of rows (scalar registers only) whose extent ends with the
    // level's d rows, so that rows beyond d read as zero, and one constant lane offset per block.
    float w[2][KSTEPS], bm[2];
    const int fcol[2] = {min(comp0 + col, F - 1), min(comp0 + 32 + col, F - 1)};
    const int w_lane_offset[2] = {4 * (half * F + fcol[0]), 4 * (half * F + fcol[1])};
    auto fetch_w = [&](const float *wm, int m, int cb) {
        // the descriptors advance by two rows per step from values the compiler cannot hoist out of the
        // level loop (kept there, 3 K scalar registers would be spilled)
        int pair_bytes = 2 * F * 4, left = d * F * 4;
        asm volatile("" : "+s"(pair_bytes), "+s"(left));
        const char *base = reinterpret_cast<const char *>(wm);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const __amdgpu_buffer_rsrc_t rows = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<char *>(base), (short)0, left, kRawBufferWord3);
            w[cb][kk] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rows, w_lane_offset[cb], 0, 0));
            const int adv = min(pair_bytes, left);
            base += adv;
            left -= adv;
        }
        bm[cb] = bias[(int64_t)m * F + fcol[cb]];
    };
    fetch_w(W, 0, 0);
    fetch_w(W, 0, 1);
    fetch_tile(0);
    put_tile(xs);
    __syncthreads();
    float *my_tile = tile[wave];
    int cur = 0;
    for (int64_t t0 = 0; t0 < L; t0 += kRows, cur ^= 1) {
        const int nrow = (int)min((int64_t)kRows, L - t0);
        const bool more = t0 + kRows < L;
        if (more) fetch_tile(t0 + kRows);
        const float *xt = xs + cur * (kRows * XS) + col * XS + half;
        float xa[kKeepX ? KSTEPS : 1];
        if (kKeepX) {
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) xa[kk] = xt[2 * kk];
        }
        float E[kRows];
        for (int m = 0; m < M; ++m) {
            const int mn = m + 1 == M ? 0 : m + 1;
            const float *wn = W + (int64_t)mn * d * F;
            // per block of 32 components: projection, then the next level's W columns are requested, then the
            // cosines; lane (half, col) holds rows 8 g + 4 half + (0..3) of component col: one 16-byte store each
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KSTEPS; ++kk)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(kKeepX ? xa[kk] : xt[2 * kk], w[cb][kk], acc, 0, 0, 0);
                const float b = bm[cb];
                fetch_w(wn, mn, cb);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    floatx4 v;
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = sqrt2_cos(fmaf(acc[4 * g + j], inv_lengthscale, b));
                    *reinterpret_cast<floatx4 *>(my_tile + (32 * cb + col) * kTileStride + 8 * g + 4 * half) = v;
                    __builtin_amdgcn_sched_barrier(0);        // four cosines at a time: bounds their temporaries
                }
            }
            lds_order();
            // recurrence down the rows for this lane's component
            float a = acc_state[m][tid];
            float pc = cos_state[m][tid];
            const float *c = my_tile + lane * kTileStride;
            if (nrow == kRows) {
                if (m == 0) run_rows<true, true>(c, t0 == 0, E, a, pc, nrow);
                else run_rows<false, true>(c, t0 == 0, E, a, pc, nrow);
            } else {
                if (m == 0) run_rows<true, false>(c, t0 == 0, E, a, pc, nrow);
                else run_rows<false, false>(c, t0 == 0, E, a, pc, nrow);
            }
            acc_state[m][tid] = a;
            cos_state[m][tid] = pc;
            lds_order();
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
        constexpr size_t kStatic = sizeof(float) * (2 * kRows * ((2 * KS) | 1) + 4 * 64 * kTileStride);             \
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
