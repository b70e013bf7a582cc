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


typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kKT = 32;             // K slab
constexpr int kLdsStride = kKT + 4; // floats per LDS row: 16 consecutive rows start in distinct bank quads

// Matrix-core kernel (v_mfma_f32_32x32x2f32). Workgroup tile (64*WT) x (64*WT), four wavefronts
// in a 2x2 grid, each owning (32*WT) x (32*WT) as WT x WT blocks of 32x32. Both operands are
// K-contiguous rows, staged per K slab of 32 through LDS with float4 loads; the next slab is
// fetched into registers while the current one is multiplied.
// MFMA k-step kk of a slab uses the physical columns kk (lanes 0-31) and kk + 16 (lanes 32-63),
// the same for both operands, so that each lane reads 16 consecutive floats of its row.
// Needs 16-byte aligned bases and leading dimensions that are multiples of 4.
// SYM: PhiY is PhiX. Only the tiles on or above the diagonal are computed (blockIdx.x enumerates
// them row by row); mirror_lower_kernel fills in the rest afterwards.
// KS = 2 (small problems only, WT = 1): a second group of four wavefronts takes every other K slab with
// its own LDS staging, so that a CU that gets a single tile still has two wavefronts per SIMD; the two
// partial tiles are added through LDS at the end, in a fixed order.
template <int WT, bool SYM, int KS = 1>
__global__ __launch_bounds__(256 * KS) void gram_mfma(
    const float *__restrict__ A, int64_t Nx, int64_t lda, const float *__restrict__ B, int64_t Ny,
    int64_t ldb, int64_t K, float *__restrict__ C, int64_t ldc)
{
    constexpr int TILE = 64 * WT;               // rows of A (and of B) per workgroup
    constexpr int NLD = TILE * (kKT / 4) / 256; // float4 loads per thread per operand per slab
    __shared__ __attribute__((aligned(16))) float As_all[KS * TILE * kLdsStride];
    __shared__ __attribute__((aligned(16))) float Bs_all[KS * TILE * kLdsStride];
    __shared__ float red[KS == 2 ? 16 * 256 : 1];       // partial tile of the second K-split group
    const int group = threadIdx.x / 256;                 // K-split group (0 when KS = 1)
    float *As = As_all + group * TILE * kLdsStride, *Bs = Bs_all + group * TILE * kLdsStride;
    const int tid = threadIdx.x % 256, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int wi = wave >> 1, wj = wave & 1;
    int64_t bi = blockIdx.y, bj = blockIdx.x;
    if (SYM) {      // linear index over the upper triangle of an nt x nt tile grid -> (bi, bj >= bi)
        const int64_t nt = (Nx + TILE - 1) / TILE, idx = blockIdx.x;
        bi = (int64_t)(((double)(2 * nt + 1) - sqrt((double)(2 * nt + 1) * (double)(2 * nt + 1) - 8.0 * (double)idx)) * 0.5);
        while (bi > 0 && bi * nt - bi * (bi - 1) / 2 > idx) --bi;                 // start of row bi
        while ((bi + 1) * nt - (bi + 1) * bi / 2 <= idx) ++bi;
        bj = bi + (idx - (bi * nt - bi * (bi - 1) / 2));
    }
    const int64_t i0 = bi * TILE, j0 = bj * TILE;

    floatx16 acc[WT][WT];
#pragma unroll
    for (int a = 0; a < WT; ++a)
#pragma unroll
        for (int b = 0; b < WT; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    float4 ra[NLD], rb[NLD];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int e = tid + 256 * u;                 // float4 slot inside the slab tile
            const int r = e / (kKT / 4), c4 = e % (kKT / 4);
            const int64_t k = k0 + 4 * c4;
            float4 va = make_float4(0.f, 0.f, 0.f, 0.f), vb = va;
            if (k < K) {
                if (i0 + r < Nx) va = *reinterpret_cast<const float4 *>(A + (i0 + r) * lda + k);
                if (j0 + r < Ny) vb = *reinterpret_cast<const float4 *>(B + (j0 + r) * ldb + k);
                if (k + 3 >= K) {                        // columns beyond K hold padding, not data
                    if (k + 1 >= K) { va.y = 0.f; vb.y = 0.f; }
                    if (k + 2 >= K) { va.z = 0.f; vb.z = 0.f; }
                    va.w = 0.f; vb.w = 0.f;
                }
            }
            ra[u] = va;
            rb[u] = vb;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int e = tid + 256 * u;
            const int r = e / (kKT / 4), c4 = e % (kKT / 4);
            *reinterpret_cast<float4 *>(&As[r * kLdsStride + 4 * c4]) = ra[u];
            *reinterpret_cast<float4 *>(&Bs[r * kLdsStride + 4 * c4]) = rb[u];
        }
    };

    // group g takes slabs g, g + KS, ...; a slab past the end is fetched as zeros, so that every group
    // runs the same number of iterations (the barriers are workgroup-wide)
    fetch((int64_t)group * kKT);
    for (int64_t kb = 0; kb < K; kb += (int64_t)KS * kKT) {
        const int64_t k0 = kb + (int64_t)group * kKT;
        __syncthreads();                                 // previous slab fully consumed
        stage();
        __syncthreads();
        if (kb + (int64_t)KS * kKT < K) fetch(k0 + (int64_t)KS * kKT);
        // this lane's 16 columns of each of its rows: physical columns 16*half .. 16*half+15
        float4 fa[WT][4], fb[WT][4];
#pragma unroll
        for (int t = 0; t < WT; ++t)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                fa[t][c] = *reinterpret_cast<const float4 *>(&As[((wi * WT + t) * 32 + col) * kLdsStride + 16 * half + 4 * c]);
                fb[t][c] = *reinterpret_cast<const float4 *>(&Bs[((wj * WT + t) * 32 + col) * kLdsStride + 16 * half + 4 * c]);
            }
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int a = 0; a < WT; ++a)
#pragma unroll
                    for (int b = 0; b < WT; ++b) {
                        const float av = e == 0 ? fa[a][c].x : e == 1 ? fa[a][c].y : e == 2 ? fa[a][c].z : fa[a][c].w;
                        const float bv = e == 0 ? fb[b][c].x : e == 1 ? fb[b][c].y : e == 2 ? fb[b][c].z : fb[b][c].w;
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[a][b], 0, 0, 0);
                    }
    }
    if constexpr (KS == 2) {                            // group 1 hands its partial tile to group 0
        static_assert(WT == 1 || KS == 1, "the K split is for the single-block tile only");
        __syncthreads();
        if (group == 1) {
#pragma unroll
            for (int v = 0; v < 16; ++v) red[v * 256 + tid] = acc[0][0][v];
        }
        __syncthreads();
        if (group == 1) return;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[0][0][v] += red[v * 256 + tid];
    }
    // result layout of a 32x32 block: lane holds column lane%32 and rows 8q + 4*(lane/32) + i
#pragma unroll
    for (int a = 0; a < WT; ++a)
#pragma unroll
        for (int b = 0; b < WT; ++b) {
            const int64_t j = j0 + (wj * WT + b) * 32 + col;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t i = i0 + (wi * WT + a) * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                if (i < Nx && j < Ny) C[i * ldc + j] = acc[a][b][v];
            }
        }
}

// Copies the part of a symmetric matrix above the diagonal to the part below it, 32x32 tiles
// transposed through LDS so that both the reads and the writes are coalesced.
__global__ __launch_bounds__(256) void mirror_lower_kernel(float *__restrict__ C, int64_t N, int64_t ldc)
{
    __shared__ float t[32][33];
    const int64_t ti = blockIdx.y, tj = blockIdx.x;
    if (tj < ti) return;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int r = ty; r < 32; r += 8) {
        const int64_t i = ti * 32 + r, j = tj * 32 + tx;
        t[r][tx] = (i < N && j < N) ? C[i * ldc + j] : 0.f;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int64_t i = tj * 32 + r, j = ti * 32 + tx;       // destination (i, j) = source (j, i)
        if (i < N && j < N && i > j) C[i * ldc + j] = t[tx][r];
    }
}

}  // namespace

hipError_t launch_gram(const float *PhiX, int64_t Nx, int64_t ldx, const float *PhiY, int64_t Ny,
                       int64_t ldy, int64_t ncols, float *K, int64_t ldk, hipStream_t stream)
{
    if (Nx == 0 || Ny == 0) return hipSuccess;
    const bool aligned = ldx % 4 == 0 && ldy % 4 == 0 && reinterpret_cast<uintptr_t>(PhiX) % 16 == 0 &&
                         reinterpret_cast<uintptr_t>(PhiY) % 16 == 0;
    if (aligned) {
        const int64_t big_tiles = ((Nx + 127) / 128) * ((Ny + 127) / 128);
        // worth it once the upper triangle alone fills the chip twice over (64-row tiles)
        const int64_t nt64 = (Nx + 63) / 64;
        const bool symmetric = PhiX == PhiY && Nx == Ny && ldx == ldy && nt64 * (nt64 + 1) / 2 >= 512;
        if (symmetric) {        // K = PhiX PhiX^T: upper triangle on the matrix cores, then mirrored
            const bool big = big_tiles >= 1024;
            const int64_t nt = (Nx + (big ? 127 : 63)) / (big ? 128 : 64);
            const int64_t tiles = nt * (nt + 1) / 2;
            if (tiles > 0x7fffffffLL || (Nx + 31) / 32 > 65535) return hipErrorInvalidValue;
            if (big)
                hipLaunchKernelGGL((gram_mfma<2, true>), dim3((unsigned)tiles), dim3(256), 0, stream, PhiX, Nx, ldx,
                                   PhiY, Ny, ldy, ncols, K, ldk);
            else
                hipLaunchKernelGGL((gram_mfma<1, true>), dim3((unsigned)tiles), dim3(256), 0, stream, PhiX, Nx, ldx,
                                   PhiY, Ny, ldy, ncols, K, ldk);
            const unsigned nm = (unsigned)((Nx + 31) / 32);
            hipLaunchKernelGGL(mirror_lower_kernel, dim3(nm, nm), dim3(256), 0, stream, K, Nx, ldk);
        } else if (big_tiles >= 512) {
            dim3 g((unsigned)((Ny + 127) / 128), (unsigned)((Nx + 127) / 128));
            hipLaunchKernelGGL((gram_mfma<2, false>), g, dim3(256), 0, stream, PhiX, Nx, ldx, PhiY, Ny, ldy, ncols, K, ldk);
        } else {
            dim3 g((unsigned)((Ny + 63) / 64), (unsigned)((Nx + 63) / 64));
            const int64_t small_tiles = (int64_t)g.x * g.y;
            if (small_tiles <= 512 && ncols >= 256)     // at most two tiles per CU: split K inside the workgroup
                hipLaunchKernelGGL((gram_mfma<1, false, 2>), g, dim3(512), 0, stream, PhiX, Nx, ldx, PhiY, Ny, ldy,
                                   ncols, K, ldk);
            else
                hipLaunchKernelGGL((gram_mfma<1, false>), g, dim3(256), 0, stream, PhiX, Nx, ldx, PhiY, Ny, ldy,
                                   ncols, K, ldk);
        }
        return hipGetLastError();
    }
    dim3 grid((unsigned)((Ny + kTile - 1) / kTile), (unsigned)((Nx + kTile - 1) / kTile));
    hipLaunchKernelGGL(gram_generic, grid, dim3(256), 0, stream, PhiX, Nx, ldx, PhiY, Ny, ldy, ncols, K, ldk);
    return hipGetLastError();
}

}  // namespace rfsf
