// Joining the pieces of sequences that were cut in time (few, long sequences: one workgroup per sequence
// would leave most of the chip idle; Sec. 4 runs 10 sequences of up to 1e5 points).
//
// Level m of RFSF-TS (Sec. 3.5, eq. (ts_rec), p = 1) is the count sketch of the sum over i1 < ... < im of the
// tensor product of the increments d_1[i1], ..., d_m[im], tensor position k sketched with hash/sign pair k;
// the sketch of a tensor product is the circular convolution of the factors' sketches, a product bin by bin
// after the transform. For a sequence x followed by a sequence y the strictly increasing index tuples split
// by how many indices fall into x, so per bin
//     A^{(1..m)}(x y) = A^{(1..m)}(y) + A^{(1..m)}(x) + sum_{j=1}^{m-1} A^{(1..j)}(x) A^{(j+1..m)}(y),
// where A^{(a..b)} is the accumulator of the recurrence run with the sketches of positions a .. b. The sketch
// kernel is therefore launched on every piece once per first position a = 1 .. M (levels a .. M of the
// increment rows, accumulators written out instead of features), this kernel folds the pieces of a sequence
// together from left to right, bin by bin, and a last launch of the sketch kernel turns the joined accumulators
// into features.
#include "rfsf_internal.h"

namespace rfsf {
namespace {

__device__ __forceinline__ float2 cmadd(float2 a, float2 b, float2 c)      // a * b + c
{
    return make_float2(fmaf(a.x, b.x, fmaf(-a.y, b.y, c.x)), fmaf(a.x, b.y, fmaf(a.y, b.x, c.y)));
}

// One thread per (sequence, bin). src.rows[a]: rows (sequence * pieces + piece) of M-a levels of `bins` numbers.
// The piece's M(M+1)/2 numbers are loaded one piece ahead of their use.
template <int M>
__global__ __launch_bounds__(256) void join_pieces_kernel(PieceRows src, int64_t n_seq, int pieces, int bins,
                                                          float2 *__restrict__ joined)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n = g / bins;
    if (n >= n_seq) return;
    const int f = (int)(g - n * bins);
    float2 A[M];
#pragma unroll
    for (int m = 0; m < M; ++m) A[m] = make_float2(0.f, 0.f);
    float2 B[M][M], Bn[M][M];               // [a][l]: first position a+1, levels a+1 .. a+1+l
    auto fetch = [&](float2 (&dst)[M][M], int s) {
        const int64_t v = n * pieces + s;
#pragma unroll
        for (int a = 0; a < M; ++a)
#pragma unroll
            for (int l = 0; l < M - a; ++l) dst[a][l] = src.rows[a][(v * (M - a) + l) * bins + f];
    };
    fetch(Bn, 0);
    for (int s = 0; s < pieces; ++s) {
#pragma unroll
        for (int a = 0; a < M; ++a)
#pragma unroll
            for (int l = 0; l < M - a; ++l) B[a][l] = Bn[a][l];
        if (s + 1 < pieces) fetch(Bn, s + 1);
        // descending levels: the lower levels are still those of the part joined so far
#pragma unroll
        for (int m = M - 1; m >= 0; --m) {
            float2 acc = make_float2(A[m].x + B[0][m].x, A[m].y + B[0][m].y);
#pragma unroll
            for (int j = 1; j <= m; ++j) acc = cmadd(A[j - 1], B[j][m - j], acc);
            A[m] = acc;
        }
    }
#pragma unroll
    for (int m = 0; m < M; ++m) joined[(n * M + m) * bins + f] = A[m];
}

}  // namespace

hipError_t launch_join_pieces(const PieceRows &pieces_of_start, int64_t n_seq, int pieces, int M, int bins,
                              float2 *joined, hipStream_t stream)
{
    if (n_seq == 0) return hipSuccess;
    if (pieces < 1 || bins < 1) return hipErrorInvalidValue;
    const int64_t blocks = (n_seq * bins + 255) / 256;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    switch (M) {
#define RFSF_JOIN_CASE(LEVELS)                                                                                        \
        case LEVELS:                                                                                                  \
            hipLaunchKernelGGL(join_pieces_kernel<LEVELS>, grid, dim3(256), 0, stream, pieces_of_start, n_seq, pieces, bins, \
                               joined);                                                                               \
            break;
        RFSF_JOIN_CASE(2) RFSF_JOIN_CASE(3) RFSF_JOIN_CASE(4) RFSF_JOIN_CASE(5) RFSF_JOIN_CASE(6) RFSF_JOIN_CASE(7)
        RFSF_JOIN_CASE(8)
#undef RFSF_JOIN_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace rfsf
