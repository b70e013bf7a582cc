// Steps 1-2 of the RFSF-TS path: per-level random Fourier features of every time point
// (Sec. 3.1, eq. (rff); W = Z / bandwidth as in the appendix class RandomFourierFeatures)
// and their increments along time (the factors nabla phi_m of Sec. 3.2, eq. (rfsf)).
#include "rfsf_internal.h"
#include "sincos.h"

// The increments are written once and read once, by the next kernel, long after they have left the caches:
// non-temporal stores (measured: the projection kernel of Large 8.2 -> 6.4 ms, Long 3 % faster, Medium unchanged;
// on Small, which would fit the last-level cache, the producer loses what the consumer gains).
typedef float rfsf_float2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_stream(float *p, float a, float b)
{
    rfsf_float2v v = {a, b};
    __builtin_nontemporal_store(v, reinterpret_cast<rfsf_float2v *>(p));
}

namespace rfsf {
namespace {

// The same, times `scale`, with the scale folded into the polynomial coefficients (no extra
// multiplies): sc = {scale, -scale/2, scale*c1, scale*c2, scale*c3} for the cosine, and the sine
// polynomial is evaluated on r*scale.
struct ScaledCoeffs { float one, half, c1, c2, c3; };
__device__ __forceinline__ ScaledCoeffs scaled_coeffs(float scale)
{
    return {scale, -0.5f * scale, 4.166664568298827e-2f * scale, -1.388731625493765e-3f * scale,
            2.443315711809948e-5f * scale};
}
__device__ __forceinline__ void sincos_scaled(float x, const ScaledCoeffs &k, float &s, float &c)
{
    const float kf = rintf(x * 0.636619772367581343f);
    float r = fmaf(-kf, 1.57079637050628662109375f, x);
    r = fmaf(-kf, -4.37113900018624283e-8f, r);
    const float r2 = r * r;
    const float rs = r * k.one;
    const float ps = fmaf(r2, fmaf(r2, -1.9515295891e-4f, 8.3321608736e-3f), -1.6666654611e-1f);
    const float S = fmaf(rs * r2, ps, rs);
    const float pc = fmaf(r2, fmaf(r2, k.c3, k.c2), k.c1);
    const float C = fmaf(r2 * r2, pc, fmaf(k.half, r2, k.one));
    const int q = (int)kf;
    const float ss = (q & 1) ? C : S;
    const float cc = (q & 1) ? S : C;
    s = __uint_as_float(__float_as_uint(ss) ^ (((unsigned)q & 2u) << 30));
    c = __uint_as_float(__float_as_uint(cc) ^ ((((unsigned)q + 1u) & 2u) << 30));
}

constexpr int kRowsPerTile = 32;

// Epilogue shared by the matrix-core kernels: sin/cos of the 16 angles a lane holds (rows
// 8q + 4*half + i of the tile, one frequency), their time difference and the stores, one block of
// four rows at a time so that stores are spread between the arithmetic. The row above a block comes
// from the partner half-wavefront (its block q for the upper half, q-1 for the lower half) or, for
// the first block of the lower half, from the previous tile (carry).
// Row layout (PAIRED = false): increment k = phi(row k+1) - phi(row k) is stored at row k, scalar base +
// 32-bit lane offset, one predicate per row.
template <typename AngleOf>
__device__ __forceinline__ void sincos_difference_store(
    AngleOf angle, const ScaledCoeffs &coeffs, float &carry_c, float &carry_s, int half, bool f_ok, int nrow,
    int64_t gt, int64_t g0, int64_t rf, int F, float *__restrict__ level_base, int f)
{
    // One store path for every tile: scalar base + 32-bit lane offset. The first row of a range has no
    // increment to store (it belongs to the previous range) and rows past the end of the range do not
    // exist; both cases are lane-uniform per row and folded into one predicate per store.
    float *cos_base = level_base + (gt - 1) * rf;               // uniform (gt = g0: row -1 is never stored)
    float *sin_base = cos_base + F;
    const uint32_t lane_off = (uint32_t)f + (uint32_t)(4 * half) * (uint32_t)rf;
    const int first = gt > g0 ? 0 : 1;                          // first tile row whose increment is ours
    float below_c = carry_c, below_s = carry_s;                 // lower half: partner's previous block
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float cs[4], sn[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) sincos_scaled(angle(4 * q + i), coeffs, sn[i], cs[i]);
        const float pc = __shfl_xor(cs[3], 32), ps = __shfl_xor(sn[3], 32);
        const float up_c = half ? pc : below_c, up_s = half ? ps : below_s;
        below_c = pc;
        below_s = ps;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float dc = cs[i] - (i ? cs[i - 1] : up_c);
            const float ds = sn[i] - (i ? sn[i - 1] : up_s);
            const int r = 8 * q + 4 * half + i;
            if (f_ok && r >= first && r < nrow) {
                const uint32_t off = lane_off + (uint32_t)(8 * q + i) * (uint32_t)rf;
                cos_base[off] = dc;
                sin_base[off] = ds;
            }
        }
    }
    carry_c = below_c;      // row 31 of this tile as seen by the lower half (unused by the upper half)
    carry_s = below_s;
}

// Pair layout: increments 2P and 2P+1 of a coordinate are stored next to each other as a float2 at
// ((P * M + m) * 2F + a), the form in which the tuned consumer loads them straight into LDS as the real and
// imaginary parts of one transform input. Tile row r is row gt + r of the (padded) row space and its increment
// has index k = gt - 1 + r with gt - 1 even, so a lane's rows i = 0,1 and i = 2,3 form pairs. A pair is stored
// when its even index lies in [k_lo, k_hi].
template <typename AngleOf>
__device__ __forceinline__ void sincos_difference_store_pairs(
    AngleOf angle, const ScaledCoeffs &coeffs, float &carry_c, float &carry_s, int half, bool f_ok,
    int64_t gt, int64_t k_lo, int64_t k_hi, int64_t pair_floats, int F, float *__restrict__ level_base, int f)
{
    const int64_t k_tile = gt - 1;                                  // even; may be -2 for the very first tile
    float *cos_base = level_base + (k_tile / 2) * pair_floats;      // uniform; pair_floats = M * 4F
    float *sin_base = cos_base + 2 * F;
    const uint32_t lane_off = 2u * (uint32_t)f + (uint32_t)(2 * half) * (uint32_t)pair_floats;
    float below_c = carry_c, below_s = carry_s;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float cs[4], sn[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) sincos_scaled(angle(4 * q + i), coeffs, sn[i], cs[i]);
        const float pc = __shfl_xor(cs[3], 32), ps = __shfl_xor(sn[3], 32);
        const float up_c = half ? pc : below_c, up_s = half ? ps : below_s;
        below_c = pc;
        below_s = ps;
        float dc[4], ds[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dc[i] = cs[i] - (i ? cs[i - 1] : up_c);
            ds[i] = sn[i] - (i ? sn[i - 1] : up_s);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t k0 = k_tile + 8 * q + 4 * half + 2 * j;  // lane-uniform per half-wavefront
            if (f_ok && k0 >= k_lo && k0 <= k_hi) {
                const uint32_t off = lane_off + (uint32_t)(4 * q + j) * (uint32_t)pair_floats;
                store_stream(cos_base + off, dc[2 * j], dc[2 * j + 1]);
                store_stream(sin_base + off, ds[2 * j], ds[2 * j + 1]);
            }
        }
    }
    carry_c = below_c;
    carry_s = below_s;
}

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


// Row of X behind row G of the padded row space (Lp rows per sequence, Lp = L rounded up to even): rows past a
// sequence's last point and rows outside the batch are redirected to the nearest existing point; the
// increments they produce are never read.
__device__ __forceinline__ int64_t padded_row_to_x_row(int64_t G, int64_t rows_pad, int64_t L, int64_t Lp)
{
    G = G < 0 ? 0 : (G >= rows_pad ? rows_pad - 1 : G);
    const int64_t n = G / Lp, t = G - n * Lp;
    return n * L + (t < L ? t : L - 1);
}
// The same without a 64-bit division per call: (n_base, t_base) are sequence and time point of row G_base
// (computed once per workgroup) and G - G_base is small (a workgroup walks 256 rows).
struct PaddedRowBase { int64_t G, n, t; };
__device__ __forceinline__ PaddedRowBase padded_row_base(int64_t G, int64_t rows_pad, int64_t Lp)
{
    G = G < 0 ? 0 : (G >= rows_pad ? rows_pad - 1 : G);
    const int64_t n = G / Lp;
    return {G, n, G - n * Lp};
}
__device__ __forceinline__ int64_t padded_row_to_x_row(int64_t G, const PaddedRowBase &b, int64_t rows_pad, int64_t L,
                                                       int64_t Lp)
{
    G = G < b.G ? b.G : (G >= rows_pad ? rows_pad - 1 : G);
    if (Lp == L) return G;                                     // even L: the padded row space is the row space of X
    int64_t t = b.t + (G - b.G), n = b.n;                      // G - b.G < 512
    if (Lp >= 512) {
        if (t >= Lp) { t -= Lp; ++n; }
    } else {
        const int q = (int)t / (int)Lp;
        t -= (int64_t)q * Lp;
        n += q;
    }
    return n * L + (t < L ? t : L - 1);
}

// The vector-ALU kernel in the pair layout (see sincos_difference_store_pairs), signs applied: a workgroup
// owns increments k_lo .. k_lo + 253 of the padded row space.
__global__ __launch_bounds__(256) void rff_increments_valu_pairs(
    const float *__restrict__ X, const float *__restrict__ W, const float *__restrict__ sign, float inv_lengthscale,
    float scale, int64_t rows_pad, int64_t L, int64_t Lp, int d, int M, int F, float *__restrict__ dphi)
{
    extern __shared__ float xs[];                     // kRowsPerTile * d
    const int fblocks = (F + 255) / 256;
    const int m = blockIdx.y / fblocks;
    const int a = (blockIdx.y % fblocks) * 256 + threadIdx.x;
    const bool active = a < F;
    const int64_t k_lo = (int64_t)blockIdx.x * 254;
    const int64_t k_hi = min(k_lo + 253, rows_pad - 1);                // odd: whole pairs
    const float *Wm = W + (int64_t)m * d * F;
    const int64_t pair_floats = (int64_t)M * 4 * F;
    const float sc = active && sign && sign[(int64_t)m * 2 * F + a] < 0.f ? -scale : scale;
    const float ss = active && sign && sign[(int64_t)m * 2 * F + F + a] < 0.f ? -scale : scale;
    float pc = 0.f, ps = 0.f, hold_c = 0.f, hold_s = 0.f;
    // phi of rows k_lo .. k_hi + 1; increment k = phi(k+1) - phi(k)
    for (int64_t gt = k_lo; gt <= k_hi + 1; gt += kRowsPerTile) {
        const int nrow = (int)min((int64_t)kRowsPerTile, k_hi + 1 - gt + 1);
        __syncthreads();
        for (int i = threadIdx.x; i < nrow * d; i += 256) {
            const int r = i / d, c = i - r * d;
            xs[i] = X[padded_row_to_x_row(gt + r, rows_pad, L, Lp) * d + c];
        }
        __syncthreads();
        if (!active) continue;
        for (int r = 0; r < nrow; ++r) {
            float acc = 0.f;
            for (int c = 0; c < d; ++c) acc = fmaf(xs[r * d + c], Wm[(int64_t)c * F + a], acc);
            float s, co;
            sincos_reduced(acc * inv_lengthscale, s, co);
            s *= ss;
            co *= sc;
            const int64_t k = gt + r - 1;             // increment that ends at this row
            if (k >= k_lo) {
                if (k & 1) {
                    float *dst = dphi + ((k / 2) * M + m) * 4 * F;
                    *reinterpret_cast<float2 *>(dst + 2 * a) = make_float2(hold_c, co - pc);
                    *reinterpret_cast<float2 *>(dst + 2 * (F + a)) = make_float2(hold_s, s - ps);
                } else {
                    hold_c = co - pc;
                    hold_s = s - ps;
                }
            }
            pc = co;
            ps = s;
        }
    }
    (void)pair_floats;
}


typedef float floatx16 __attribute__((ext_vector_type(16)));

// Matrix-core kernel (fp32 operands). A workgroup of four wavefronts owns 128 frequencies of
// one level and a range of flattened rows; wavefront w owns frequencies 32w..32w+31. Per tile
// of 32 rows, theta[32 rows x 32 freq] = X_tile[32 x d] * W[d x 32] is accumulated with
// v_mfma_f32_32x32x2f32 (A = rows x channels from LDS, B = channels x frequencies held in
// registers for the whole row range). In the result a lane holds one frequency (lane % 32)
// and rows 8q + 4*(lane/32) + i, q,i = 0..3, so the time difference is local except at the
// 4-row boundaries, where the two half-wavefronts exchange one value per block of rows.
// PAIRED: pair layout with the CountSketch signs applied (for the tuned consumer). `rows` is then the padded
// row count n_seq * Lp, a workgroup owns increments g0 .. g0 + 253 (g0 = 254 * range, even) and its tiles start
// one row early, at the odd row g0 - 1, so that a lane's four rows split into two whole pairs. Signs cost
// nothing: flipping both coordinates of a frequency is a negative scale, flipping the sine alone is a negated
// frequency vector (sin(-x) = -sin x, cos(-x) = cos x), flipping the cosine alone is both.
template <int KSTEPS, bool PAIRED>     // ceil(d / 2) padded: channels 2*KSTEPS
__global__ __launch_bounds__(256) void rff_increments_mfma(
    const float *__restrict__ X, const float *__restrict__ W, const float *__restrict__ sign, float inv_lengthscale,
    float scale, int64_t rows, int64_t L, int64_t Lp, int d, int M, int F, int64_t rows_per_block,
    float *__restrict__ dphi)
{
    constexpr int KP = 2 * KSTEPS;              // padded channel count
    constexpr int XS = KP | 1;                  // odd LDS row stride: conflict-free A reads
    __shared__ float xs[2 * kRowsPerTile * XS];
    // Block order: the (level, frequency slab) index runs fastest, so that the workgroups that write the
    // same rows are dispatched together, which keeps the writes of one DRAM page close in time (also with
    // few slabs: four slabs of 1000 short sequences run 17 % faster this way than row range first).
    const int fblocks = (F + 127) / 128;
    const int nslab = M * fblocks;
    const int slab = (int)(blockIdx.x % nslab);
    const int64_t range = blockIdx.x / nslab;
    const int m = slab / fblocks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int f = (slab % fblocks) * 128 + wave * 32 + col;           // this lane's frequency
    const bool f_ok = f < F;
    const int64_t g0 = range * rows_per_block;
    // last row whose phi we need (PAIRED: row `rows` does not exist and is redirected)
    const int64_t g1 = PAIRED ? min(rows, g0 + rows_per_block) : min(rows - 1, g0 + rows_per_block);
    const int64_t rf = (int64_t)M * 2 * F;
    bool flip_c = false, flip_s = false;
    if (PAIRED && f_ok) {
        flip_c = sign[(int64_t)m * 2 * F + f] < 0.f;
        flip_s = sign[(int64_t)m * 2 * F + F + f] < 0.f;
    }
    const float wscale = (flip_c != flip_s) ? -inv_lengthscale : inv_lengthscale;

    // B operand: W[m][k][f] for k = 2*kk + half, zero beyond d or F
    float breg[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        const int k = 2 * kk + half;
        breg[kk] = (f_ok && k < d) ? W[((int64_t)m * d + k) * F + f] * wscale : 0.f;
    }
    float carry_c = 0.f, carry_s = 0.f;         // row 31 of the previous tile (lower half-wavefront)
    float *level_base = dphi + (int64_t)m * (PAIRED ? 4 : 2) * F;     // uniform; the lane's frequency is added per store
    const ScaledCoeffs coeffs = scaled_coeffs(flip_c ? -scale : scale);
    const int64_t first_row = PAIRED ? g0 - 1 : g0;                    // row of tile row 0 of the first tile
    const PaddedRowBase row_base = PAIRED ? padded_row_base(first_row, rows, Lp) : PaddedRowBase{0, 0, 0};

    // X tiles are double-buffered in LDS: the next tile's rows are fetched into registers before the
    // current tile is processed and written to the other buffer afterwards (one barrier per tile).
    constexpr int NX = (kRowsPerTile * KP + 255) / 256;
    float xr[NX];
    auto fetch_tile = [&](int64_t gt) {
        const int nrow = (int)min((int64_t)kRowsPerTile, g1 - gt + 1);
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            const int i = threadIdx.x + 256 * u;
            const int r = i / KP, c = i - r * KP;
            if (PAIRED)
                xr[u] = (i < kRowsPerTile * KP && c < d) ? X[padded_row_to_x_row(gt + r, row_base, rows, L, Lp) * d + c] : 0.f;
            else
                xr[u] = (i < kRowsPerTile * KP && r < nrow && c < d) ? X[(gt + r) * d + c] : 0.f;
        }
    };
    auto put_tile = [&](float *buf) {
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            const int i = threadIdx.x + 256 * u;
            const int r = i / KP, c = i - r * KP;
            if (i < kRowsPerTile * KP) buf[r * XS + c] = xr[u];
        }
    };
    fetch_tile(first_row);
    put_tile(xs);
    __syncthreads();
    int cur = 0;
    for (int64_t gt = first_row; gt <= g1; gt += kRowsPerTile, cur ^= 1) {
        const int nrow = (int)min((int64_t)kRowsPerTile, g1 - gt + 1);
        const bool more = gt + kRowsPerTile <= g1;
        if (more) fetch_tile(gt + kRowsPerTile);
        const float *xt = xs + cur * (kRowsPerTile * XS);
        floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xt[col * XS + 2 * kk + half], breg[kk], acc, 0, 0, 0);

        if (PAIRED)
            sincos_difference_store_pairs([&](int v) { return acc[v]; }, coeffs, carry_c, carry_s, half, f_ok, gt, g0,
                                          min(g0 + rows_per_block - 2, rows - 2), 2 * rf, F, level_base, f);
        else
            sincos_difference_store([&](int v) { return acc[v]; }, coeffs, carry_c, carry_s, half, f_ok, nrow, gt, g0,
                                    rf, F, level_base, f);
        if (more) put_tile(xs + (cur ^ 1) * (kRowsPerTile * XS));
        __syncthreads();
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
template <int KSTEPS, bool PAIRED>     // ceil(d / 16): channels padded to 16*KSTEPS; PAIRED as in the fp32 kernel
__global__ __launch_bounds__(256) void rff_increments_mfma_bf16(
    const float *__restrict__ X, const float *__restrict__ W, const float *__restrict__ sign, float inv_lengthscale,
    float scale, int64_t rows, int64_t L, int64_t Lp, int d, int M, int F, int64_t rows_per_block,
    float *__restrict__ dphi)
{
    constexpr int KP = 16 * KSTEPS;
    constexpr int XS = KP + 8;                  // bf16 elements per LDS row (16-byte padded)
    __shared__ __attribute__((aligned(16))) uint16_t xhi[2 * kRowsPerTile * XS];
    __shared__ __attribute__((aligned(16))) uint16_t xlo[2 * kRowsPerTile * XS];
    const int fblocks = (F + 127) / 128;                              // same block order as the fp32 kernel
    const int nslab = M * fblocks;
    const int slab = (int)(blockIdx.x % nslab);
    const int64_t range = blockIdx.x / nslab;
    const int m = slab / fblocks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int f = (slab % fblocks) * 128 + wave * 32 + col;
    const bool f_ok = f < F;
    const int64_t g0 = range * rows_per_block;
    const int64_t g1 = PAIRED ? min(rows, g0 + rows_per_block) : min(rows - 1, g0 + rows_per_block);
    const int64_t rf = (int64_t)M * 2 * F;
    bool flip_c = false, flip_s = false;
    if (PAIRED && f_ok) {
        flip_c = sign[(int64_t)m * 2 * F + f] < 0.f;
        flip_s = sign[(int64_t)m * 2 * F + F + f] < 0.f;
    }
    const float wsign = (flip_c != flip_s) ? -1.0f : 1.0f;     // exact in bf16: the rounding of W is unchanged

    // B operand: lane holds W[m][16*kk + 8*half + e][f], e = 0..7, as bf16
    bf16x8 breg[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const int k = 16 * kk + 8 * half + e;
            const float w0 = (f_ok && k < d) ? W[((int64_t)m * d + k) * F + f] * wsign : 0.f;
            const float w1 = (f_ok && k + 1 < d) ? W[((int64_t)m * d + k + 1) * F + f] * wsign : 0.f;
            w[e / 2] = bf16_bits(w0) | (bf16_bits(w1) << 16);
        }
        breg[kk] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    }
    float carry_c = 0.f, carry_s = 0.f;
    float *level_base = dphi + (int64_t)m * (PAIRED ? 4 : 2) * F;     // uniform; the lane's frequency is added per store
    const ScaledCoeffs coeffs = scaled_coeffs(flip_c ? -scale : scale);
    const int64_t first_row = PAIRED ? g0 - 1 : g0;
    const PaddedRowBase row_base = PAIRED ? padded_row_base(first_row, rows, Lp) : PaddedRowBase{0, 0, 0};

    // double-buffered X tiles, as in the fp32 kernel; the split into two bf16 terms happens when a
    // tile is written to LDS
    constexpr int NX = (kRowsPerTile * KP + 255) / 256;
    constexpr int TILE = kRowsPerTile * XS;
    float xr[NX];
    auto fetch_tile = [&](int64_t gt) {
        const int nrow = (int)min((int64_t)kRowsPerTile, g1 - gt + 1);
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            const int i = threadIdx.x + 256 * u;
            const int r = i / KP, c = i - r * KP;
            if (PAIRED)
                xr[u] = (i < kRowsPerTile * KP && c < d) ? X[padded_row_to_x_row(gt + r, row_base, rows, L, Lp) * d + c] : 0.f;
            else
                xr[u] = (i < kRowsPerTile * KP && r < nrow && c < d) ? X[(gt + r) * d + c] : 0.f;
        }
    };
    auto put_tile = [&](int buf) {
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            const int i = threadIdx.x + 256 * u;
            const int r = i / KP, c = i - r * KP;
            if (i < kRowsPerTile * KP) {
                const uint32_t hi = bf16_bits(xr[u]);
                xhi[buf * TILE + r * XS + c] = (uint16_t)hi;
                xlo[buf * TILE + r * XS + c] = (uint16_t)bf16_bits(xr[u] - bf16_value(hi));
            }
        }
    };
    fetch_tile(first_row);
    put_tile(0);
    __syncthreads();
    int cur = 0;
    for (int64_t gt = first_row; gt <= g1; gt += kRowsPerTile, cur ^= 1) {
        const int nrow = (int)min((int64_t)kRowsPerTile, g1 - gt + 1);
        const bool more = gt + kRowsPerTile <= g1;
        if (more) fetch_tile(gt + kRowsPerTile);
        floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int at = cur * TILE + col * XS + 16 * kk + 8 * half;
            const bf16x8 ah = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&xhi[at]));
            const bf16x8 al = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&xlo[at]));
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, breg[kk], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, breg[kk], acc, 0, 0, 0);
        }
        if (PAIRED)
            sincos_difference_store_pairs([&](int v) { return acc[v] * inv_lengthscale; }, coeffs, carry_c, carry_s,
                                          half, f_ok, gt, g0, min(g0 + rows_per_block - 2, rows - 2), 2 * rf, F,
                                          level_base, f);
        else
            sincos_difference_store([&](int v) { return acc[v] * inv_lengthscale; }, coeffs, carry_c, carry_s, half,
                                    f_ok, nrow, gt, g0, rf, F, level_base, f);
        if (more) put_tile(cur ^ 1);
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_rff_increments(const float *X, const float *W, const float *sign, float inv_lengthscale,
                                 int64_t n_seq, int64_t L, int d, int M, int F, bool bf16,
                                 float *dphi, hipStream_t stream)
{
    const bool paired = sign != nullptr;
    const int64_t Lp = (L + 1) & ~(int64_t)1;
    const int64_t rows = paired ? n_seq * Lp : n_seq * L;
    if (rows < 2) return hipSuccess;
    // Row layout: 255 increments per workgroup (256 rows of phi = eight tiles; consecutive workgroups share one
    // row). Pair layout: 254 increments, the eight tiles start one row early; problems that would give fewer
    // than 4096 (2048) workgroups that way -- two rounds (one) of what the chip holds -- take ranges of four
    // (two) tiles instead (1000 sequences of 100 points: 0.095 -> 0.080 ms; large problems are faster with
    // eight, except that 126 increments measured 7 % faster on 10000 x 200 x 17 -- and 11 % slower on
    // 2000 x 2000 x 32 and 50000 x 64 x 64).
    int64_t rows_per_block = paired ? 254 : 255;
    if (paired) {
        const int64_t wgs = ((rows - 2) / 254 + 1) * M * ((F + 127) / 128);
        if (wgs < 2048) rows_per_block = 62;
        else if (wgs < 4096) rows_per_block = 126;
    }
    const int64_t nblk = paired ? (rows - 2) / rows_per_block + 1 : (rows - 1 + rows_per_block - 1) / rows_per_block;
    const float scale = 0.5f / sqrtf((float)F);    // the consumer's two-for-one FFT wants halved increments
    if (nblk * M * ((F + 127) / 128) > 0x7fffffffLL) return hipErrorInvalidValue;
    if (bf16) {            // the caller (API layer) has checked d <= 128
        const int fb = (F + 127) / 128;
        dim3 grid((unsigned)(nblk * M * fb));
#define RFSF_LAUNCH_BF16(KS)                                                                                     \
    do {                                                                                                         \
        if (paired)                                                                                              \
            hipLaunchKernelGGL((rff_increments_mfma_bf16<KS, true>), grid, dim3(256), 0, stream, X, W, sign,     \
                               inv_lengthscale, scale, rows, L, Lp, d, M, F, rows_per_block, dphi);              \
        else                                                                                                     \
            hipLaunchKernelGGL((rff_increments_mfma_bf16<KS, false>), grid, dim3(256), 0, stream, X, W, sign,    \
                               inv_lengthscale, scale, rows, L, Lp, d, M, F, rows_per_block, dphi);              \
    } while (0)
        if (d <= 16) RFSF_LAUNCH_BF16(1);
        else if (d <= 32) RFSF_LAUNCH_BF16(2);
        else if (d <= 64) RFSF_LAUNCH_BF16(4);
        else RFSF_LAUNCH_BF16(8);
#undef RFSF_LAUNCH_BF16
        return hipGetLastError();
    }
    if (d <= 64) {
        const int fb = (F + 127) / 128;
        dim3 grid((unsigned)(nblk * M * fb));
#define RFSF_LAUNCH_MFMA(KS)                                                                                     \
    do {                                                                                                         \
        if (paired)                                                                                              \
            hipLaunchKernelGGL((rff_increments_mfma<KS, true>), grid, dim3(256), 0, stream, X, W, sign,          \
                               inv_lengthscale, scale, rows, L, Lp, d, M, F, rows_per_block, dphi);              \
        else                                                                                                     \
            hipLaunchKernelGGL((rff_increments_mfma<KS, false>), grid, dim3(256), 0, stream, X, W, sign,         \
                               inv_lengthscale, scale, rows, L, Lp, d, M, F, rows_per_block, dphi);              \
    } while (0)
        if (d <= 4) RFSF_LAUNCH_MFMA(2);
        else if (d <= 8) RFSF_LAUNCH_MFMA(4);
        else if (d <= 18) RFSF_LAUNCH_MFMA(9);
        else if (d <= 32) RFSF_LAUNCH_MFMA(16);
        else RFSF_LAUNCH_MFMA(32);
#undef RFSF_LAUNCH_MFMA
        return hipGetLastError();
    }
    const int fblocks = (F + 255) / 256;
    if ((int64_t)M * fblocks > 65535) return hipErrorInvalidValue;
    if (paired) {
        const int64_t nb = (rows - 2) / 254 + 1;
        if (nb > 0x7fffffffLL) return hipErrorInvalidValue;
        dim3 grid((unsigned)nb, (unsigned)(M * fblocks));
        hipLaunchKernelGGL(rff_increments_valu_pairs, grid, dim3(256), sizeof(float) * kRowsPerTile * d, stream,
                           X, W, sign, inv_lengthscale, scale, rows, L, Lp, d, M, F, dphi);
        return hipGetLastError();
    }
    dim3 grid((unsigned)nblk, (unsigned)(M * fblocks));
    hipLaunchKernelGGL(rff_increments_valu, grid, dim3(256), sizeof(float) * kRowsPerTile * d, stream,
                       X, W, inv_lengthscale, scale, rows, d, M, F, rows_per_block, dphi);
    return hipGetLastError();
}

}  // namespace rfsf
