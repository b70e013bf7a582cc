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

// Tile order of the large-problem kernel. The hardware deals consecutive workgroup ids round-robin to the
// eight XCDs, each with its own L2. Tiles are therefore first put in a locality order -- strips of eight tile
// rows, inside a strip column by column -- and that list is cut into eight equal contiguous pieces, one per
// XCD: the 64 or so tiles an XCD has in flight then form an 8 x 8 block that shares eight row panels and
// eight column panels through its L2, and every XCD gets the same number of tiles (to within one).
// SYM: only tiles on or above the diagonal exist; a strip starts with its triangular part.
struct TileCoord { int64_t bi, bj; };
constexpr int kStrip = 8;
template <bool SYM>
__device__ __forceinline__ TileCoord tile_of_rank(int64_t rank, int64_t nti, int64_t ntj)
{
    if (!SYM) {
        const int64_t full = kStrip * ntj, I = rank / full, r = rank - I * full;
        const int64_t h = nti - kStrip * I < kStrip ? nti - kStrip * I : kStrip;
        return {kStrip * I + r % h, r / h};
    }
    int64_t I = 0;
    for (;; ++I) {
        const int64_t h = nti - kStrip * I < kStrip ? nti - kStrip * I : kStrip;
        const int64_t cnt = h * (h + 1) / 2 + h * (nti - kStrip * I - h);
        if (rank < cnt) break;
        rank -= cnt;
    }
    const int64_t h = nti - kStrip * I < kStrip ? nti - kStrip * I : kStrip, tri = h * (h + 1) / 2;
    if (rank < tri) {                       // column c of the triangle holds rows 0..c
        int64_t c = 0;
        while (rank >= c + 1) { rank -= c + 1; ++c; }
        return {kStrip * I + rank, kStrip * I + c};
    }
    rank -= tri;
    return {kStrip * I + rank % h, kStrip * I + h + rank / h};
}

// Matrix-core kernel for large problems: 128 x 128 tile, four wavefronts 2 x 2, v_mfma_f32_32x32x2f32, K slabs
// of 32 in two LDS buffers. While slab s is multiplied out of one buffer, slab s+1 is loaded from global memory
// straight into the other one (global_load_lds_dwordx4: lane i of a wavefront deposits its 16 bytes at
// LDS base + 16 i, no register and no LDS-write instruction involved -- measured here, LDS writes issued by
// the wavefronts cost 11 % of the matrix rate, because they hold the issue port the matrix instructions need).
// One barrier per slab separates the two roles of a buffer.
// LDS layout of one operand in one buffer: 128 rows x 8 chunks of 16 bytes, unpadded; chunk slot p of row r
// holds columns 4 (p ^ s(r)) .. +3 of the slab, s(r) = (r / 2) mod 8. The XOR makes the fragment reads
// (16 consecutive rows, same chunk) hit 16 distinct 16-byte positions of the 256-byte bank row, and a direct
// load can produce it because each lane chooses which global chunk it fetches. MFMA k-step (c, e) uses column
// 4c + e in lanes 0-31 and 16 + 4c + e in lanes 32-63, for both operands.
// The last slab, if K is no multiple of 32, goes through registers so that columns beyond K can be zeroed.
constexpr int kBigTile = 128;
constexpr int kBigOperand = kBigTile * kKT;                 // floats of one operand in one buffer

// Fragments of one lane for k-groups c = C0 .. C0+1 of a staged slab: row (wi or wj)*64 + 32 t + col of each
// operand, chunk 4 half + c in slot (4 half + c) ^ s(row).
struct BigFrag { float4 a[2][2], b[2][2]; };           // [c - C0][t]
template <int C0>
__device__ __forceinline__ void big_read(const float *__restrict__ rd, int frag_a, int frag_b, int half, int fsw, BigFrag &f)
{
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int slot = 4 * ((4 * half + C0 + c) ^ fsw);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f.a[c][t] = *reinterpret_cast<const float4 *>(&rd[frag_a + t * 32 * kKT + slot]);
            f.b[c][t] = *reinterpret_cast<const float4 *>(&rd[frag_b + t * 32 * kKT + slot]);
        }
    }
}
// 16 matrix instructions on k-group c of a fragment pair
__device__ __forceinline__ void big_mfma16(const BigFrag &f, int c, floatx16 (&acc)[2][2])
{
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const float4 &fa = f.a[c][a], &fb = f.b[c][b];
                const float av = e == 0 ? fa.x : e == 1 ? fa.y : e == 2 ? fa.z : fa.w;
                const float bv = e == 0 ? fb.x : e == 1 ? fb.y : e == 2 ? fb.z : fb.w;
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[a][b], 0, 0, 0);
            }
}

// Direct loads of one full slab (columns k0 .. k0+31) into `wr`: wavefront `wave` fills rows 32u + 8 wave .. +7.
__device__ __forceinline__ void big_load_direct(float *__restrict__ wr, const float *const (&pa)[4],
                                                const float *const (&pb)[4], int64_t k0, int wave)
{
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        float *dst = wr + (32 * u + 8 * wave) * kKT;        // wavefront-uniform
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(pa[u] + k0),
                                         (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(pb[u] + k0),
                                         (__attribute__((address_space(3))) void *)(dst + kBigOperand), 16, 0, 0);
    }
}

// One steady-state step, software-pipelined across the barrier: on entry `f01` holds the fragments of
// k-groups 0, 1 of the slab in `rd`. The next slab's direct loads go out first and have three quarters of the
// step to land; the barrier sits before the last 16 matrix instructions, so that the first LDS reads of the next
// slab (into `f01` again) run under them instead of stalling the matrix pipe after the barrier. `rd` and `wr`
// are the two distinct LDS buffers; telling the compiler so (restrict) keeps it from waiting for the loads
// before the reads of `rd`.
__device__ __forceinline__ void big_step(const float *__restrict__ rd, float *__restrict__ wr,
                                         const float *const (&pa)[4], const float *const (&pb)[4], int64_t k_next,
                                         int wave, int frag_a, int frag_b, int half, int fsw, BigFrag &f01,
                                         floatx16 (&acc)[2][2])
{
    BigFrag f23;
    big_load_direct(wr, pa, pb, k_next, wave);
    big_read<2>(rd, frag_a, frag_b, half, fsw, f23);
    big_mfma16(f01, 0, acc);
    big_mfma16(f01, 1, acc);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);  // 4 matrix instructions
        __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);  // one direct load of the next slab
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read of k-groups 2, 3
    }
    big_mfma16(f23, 0, acc);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();                                        // next slab complete, this one read by everyone
    big_read<0>(wr, frag_a, frag_b, half, fsw, f01);
    big_mfma16(f23, 1, acc);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);  // one LDS read of the next slab's k-groups 0, 1
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 1);  // 2 matrix instructions
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <bool SYM>
__global__ __launch_bounds__(256, 2) void gram_mfma_big(
    const float *__restrict__ A, int64_t Nx, int64_t lda, const float *__restrict__ B, int64_t Ny,
    int64_t ldb, int64_t K, float *__restrict__ C, int64_t ldc, int64_t ntiles, int64_t per_xcd)
{
    // two buffers of [A | B][128 rows][32]; 64 KB in all (the direct loads address LDS with 16 bits)
    __shared__ __attribute__((aligned(16))) float buf0[2 * kBigOperand];
    __shared__ __attribute__((aligned(16))) float buf1[2 * kBigOperand];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, col = lane & 31;
    const int wi = wave >> 1, wj = wave & 1;
    const int64_t xcd = blockIdx.x % 8, k_in_xcd = blockIdx.x / 8;
    const int64_t rank = xcd * per_xcd + k_in_xcd;
    if (k_in_xcd >= per_xcd || rank >= ntiles) return;
    const int64_t nti = (Nx + kBigTile - 1) / kBigTile, ntj = (Ny + kBigTile - 1) / kBigTile;
    const TileCoord tc = tile_of_rank<SYM>(rank, nti, ntj);
    const int64_t i0 = tc.bi * kBigTile, j0 = tc.bj * kBigTile;

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // Loading: wavefront w fills rows 32u + 8w .. +7 (u = 0..3) of each operand; lane i covers row i/8 of those
    // and chunk slot i%8. Rows beyond the matrix are redirected to row 0: what they contribute lands in output
    // rows or columns that are never stored.
    const int lrow = 8 * wave + (lane >> 3);                 // row within a group of 32
    const int lchunk = (lane & 7) ^ ((lrow >> 1) & 7);       // global chunk that belongs in this lane's slot
    const float *pa[4], *pb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t ra_ = i0 + lrow + 32 * u, rb_ = j0 + lrow + 32 * u;
        pa[u] = A + (ra_ < Nx ? ra_ : 0) * lda + 4 * lchunk;
        pb[u] = B + (rb_ < Ny ? rb_ : 0) * ldb + 4 * lchunk;
    }
    float4 ra[4], rb[4];
    auto fetch_masked = [&](int64_t k0) {                    // through registers: columns >= K become zero
        const int64_t k = k0 + 4 * lchunk;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float4 va = make_float4(0.f, 0.f, 0.f, 0.f), vb = va;
            if (k < K) {
                va = *reinterpret_cast<const float4 *>(pa[u] + k0);
                vb = *reinterpret_cast<const float4 *>(pb[u] + k0);
                if (k + 3 >= K) {                            // columns beyond K hold padding, not data
                    if (k + 1 >= K) { va.y = 0.f; vb.y = 0.f; }
                    if (k + 2 >= K) { va.z = 0.f; vb.z = 0.f; }
                    va.w = 0.f; vb.w = 0.f;
                }
            }
            ra[u] = va;
            rb[u] = vb;
        }
    };
    auto stage_masked = [&](float *buf) {                    // the same slots the direct loads would fill
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float *dst = buf + (32 * u + 8 * wave) * kKT + 4 * lane;
            *reinterpret_cast<float4 *>(dst) = ra[u];
            *reinterpret_cast<float4 *>(dst + kBigOperand) = rb[u];
        }
    };
    const int fsw = (col >> 1) & 7;
    const int frag_a = (wi * 64 + col) * kKT, frag_b = kBigOperand + (wj * 64 + col) * kKT;
    const bool vec_store = ldc % 4 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0;    // for the mirrored stores

    const int64_t nfull = K / kKT, nslab = (K + kKT - 1) / kKT;
    if (nfull > 0) {
        big_load_direct(buf0, pa, pb, 0, wave);
    } else {
        fetch_masked(0);
        stage_masked(buf0);
    }
    __syncthreads();
    BigFrag f01, f23;
    big_read<0>(buf0, frag_a, frag_b, half, fsw, f01);
    int64_t sl = 0;
    // steady state, two slabs per trip so that each step names its buffers statically
    for (; sl + 2 < nfull; sl += 2) {
        big_step(buf0, buf1, pa, pb, (sl + 1) * kKT, wave, frag_a, frag_b, half, fsw, f01, acc);
        big_step(buf1, buf0, pa, pb, (sl + 2) * kKT, wave, frag_a, frag_b, half, fsw, f01, acc);
    }
    // the last slabs (at most two full ones and the partial one): loads through registers; `f01` holds the
    // first half of slab sl
    for (; sl < nslab; ++sl) {
        const bool more = sl + 1 < nslab;
        float *rd = (sl & 1) ? buf1 : buf0, *wr = (sl & 1) ? buf0 : buf1;
        if (more) fetch_masked((sl + 1) * kKT);
        big_read<2>(rd, frag_a, frag_b, half, fsw, f23);
        big_mfma16(f01, 0, acc);
        big_mfma16(f01, 1, acc);
        big_mfma16(f23, 0, acc);
        big_mfma16(f23, 1, acc);
        if (more) stage_masked(wr);
        __syncthreads();
        if (more) big_read<0>(wr, frag_a, frag_b, half, fsw, f01);
    }
    // result layout of a 32x32 block: lane holds column lane%32 and rows 8q + 4*(lane/32) + i
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int64_t j = j0 + (wj * 2 + b) * 32 + col;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t i = i0 + (wi * 2 + a) * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                if (i < Nx && j < Ny) C[i * ldc + j] = acc[a][b][v];
            }
            // SYM, tile above the diagonal: its mirror image below the diagonal is written from the same
            // registers (four consecutive rows of the tile are four consecutive floats of the mirrored row)
            if (SYM && tc.bi != tc.bj && j < Ny) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t i = i0 + (wi * 2 + a) * 32 + 8 * q + 4 * half;
                    float *dst = C + j * ldc + i;
                    if (i + 3 < Nx && vec_store) {
                        *reinterpret_cast<float4 *>(dst) = make_float4(acc[a][b][4 * q], acc[a][b][4 * q + 1],
                                                                       acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (i + e < Nx) dst[e] = acc[a][b][4 * q + e];
                    }
                }
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

template <bool SYM>
hipError_t launch_big(const float *PhiX, int64_t Nx, int64_t ldx, const float *PhiY, int64_t Ny, int64_t ldy,
                      int64_t ncols, float *K, int64_t ldk, int64_t tiles, hipStream_t stream)
{
    const int64_t per_xcd = (tiles + 7) / 8;
    hipLaunchKernelGGL((gram_mfma_big<SYM>), dim3((unsigned)(per_xcd * 8)), dim3(256), 0, stream, PhiX, Nx, ldx,
                       PhiY, Ny, ldy, ncols, K, ldk, tiles, per_xcd);
    return hipGetLastError();
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
            if (big) {
                const hipError_t e = launch_big<true>(PhiX, Nx, ldx, PhiY, Ny, ldy, ncols, K, ldk, tiles, stream);
                if (e != hipSuccess) return e;
            } else
                hipLaunchKernelGGL((gram_mfma<1, true>), dim3((unsigned)tiles), dim3(256), 0, stream, PhiX, Nx, ldx,
                                   PhiY, Ny, ldy, ncols, K, ldk);
            if (!big) {         // the large-tile kernel writes the mirror image itself
                const unsigned nm = (unsigned)((Nx + 31) / 32);
                hipLaunchKernelGGL(mirror_lower_kernel, dim3(nm, nm), dim3(256), 0, stream, K, Nx, ldk);
            }
        } else if (big_tiles >= 512) {
            if (big_tiles > 0x7fffffffLL - 8) return hipErrorInvalidValue;
            const hipError_t e = launch_big<false>(PhiX, Nx, ldx, PhiY, Ny, ldy, ncols, K, ldk, big_tiles, stream);
            if (e != hipSuccess) return e;
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
