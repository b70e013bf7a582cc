// Internal declarations shared by the translation units of librfsf_ts (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace rfsf {

// A launch of the tuned sketch kernels may cut every sequence into `pieces` pieces of `pairs` pairs of time
// steps each (workgroup v then owns piece v % pieces of sequence v / pieces and row v of its output), and may
// run only the first levels of increment rows that hold `row_levels` levels (the pointers to the increments
// and the tables are then advanced to the first level to run). `mode` 1: instead of the features, the
// accumulators of the recurrence (levels x bins 0 .. D/2 of the transform, complex) are written to row v of
// `spectra`; `mode` 2: no time step is run, the accumulators are read from `spectra` and turned into
// features (the final transforms).
struct TimeCut {
    int pieces, row_levels;
    int64_t pairs;
    float2 *spectra;
    int mode;
    static TimeCut whole(int64_t L, int M) { return {1, M, (L + 1) / 2, nullptr, 0}; }
};
constexpr int kMaxCutLevels = 8;                       // the tuned kernels run at most eight levels
struct PieceRows { const float2 *rows[kMaxCutLevels]; };

// Increment workspace: row g = n * L + t holds, for every level m, the 2F numbers
// phi_m(x_{t+1}) - phi_m(x_t) of sequence n; rows with t = L-1 exist but are never read.
// Element (g, m, a) sits at ((g * M + m) * 2F + a).

// Steps 1-2: random Fourier features of every time point and their time increments
// for `n_seq` sequences starting at X (already offset to the chunk), halved.
// sign == nullptr: row layout, element (g, m, a) of row g = n * L + t at ((g * M + m) * 2F + a), no signs.
// sign != nullptr ([M, 2F], the CountSketch signs): pair layout with the signs applied. With Lp = L rounded up
// to even, increment k = n * Lp + t of coordinate a sits at ((((k / 2) * M + m) * 2F + a) * 2 + k % 2): the
// two increments of a pair of consecutive time steps are one float2. n_seq * Lp * M * 2F floats in all.
hipError_t launch_rff_increments(const float *X, const float *W, const float *sign, float inv_lengthscale,
                                 int64_t n_seq, int64_t L, int d, int M, int F, bool bf16,
                                 float *dphi, hipStream_t stream);

// Steps 3-4: CountSketch, FFT-domain level recursion over time, inverse transform; writes
// (D is the transform length, a power of two; Dout <= D the number of buckets per level: equal to D,
// or smaller when the buckets are no power of two and the convolutions are linear, folded at the end)
// columns 0 .. M*D of `n_seq` rows of out (already offset to the chunk).
// `lengths` (may be null: all L) holds each sequence's own number of points, X being padded to L.
// `state` is scratch for the generic kernel: sketch_fft_scan_state_bytes (accumulators, and the work buffers
// when they do not fit in LDS).
// `table` (sketch_fft_scan_table_bytes, filled by launch_pack_tables once per call) feeds the tuned kernel.
// `cut` (tuned kernels only): how the launch cuts the sequences in time and which levels of the increment rows
// it runs; TimeCut::whole(L, M) for the plain case.
hipError_t launch_sketch_fft_scan(const float *dphi, const int32_t *hash, const float *sign,
                                  const uint32_t *table, int64_t n_seq, int64_t L, const int64_t *lengths, int M, int F,
                                  int D, int Dout, int order, float *out, int64_t ld_out, float *state,
                                  hipStream_t stream, TimeCut cut);
// Joins the pieces of a launch series that cut the sequences in time (csrc/join_pieces.hip).
// pieces_of_start.rows[a]: accumulators written by the launch that ran levels a+1 .. M (row = sequence *
// pieces + piece, M-a levels of `bins` complex numbers each). Writes M levels of `bins` numbers per sequence
// to `joined`.
hipError_t launch_join_pieces(const PieceRows &pieces_of_start, int64_t n_seq, int pieces, int M, int bins,
                              float2 *joined, hipStream_t stream);
hipError_t launch_pack_tables(const int32_t *hash, const float *sign, int M, int F, int D, int Dout,
                              uint32_t *table, hipStream_t stream);
bool sketch_fft_scan_is_tuned(int M, int F, int D);
bool sketch_fft_scan_fits(int M, int F, int D, int order);  // false: neither kernel can run it (LDS need above a CU's)
size_t sketch_fft_scan_table_bytes(int M, int F, int D);   // 0 when the generic kernel runs
size_t sketch_fft_scan_lds_bytes(int M, int F, int D);
size_t sketch_fft_scan_state_bytes(int64_t n_seq, int M, int D, int order);

// Level-0 column and zero blocks for sequences without increments (L == 1).
hipError_t launch_fill_trivial(float *out, int64_t n_seq, int64_t ld_out, int64_t ncols, hipStream_t stream);

hipError_t launch_gram(const float *PhiX, int64_t Nx, int64_t ldx, const float *PhiY, int64_t Ny,
                       int64_t ldy, int64_t ncols, float *K, int64_t ldk, hipStream_t stream);

// RFSF-DP-1D features, one fused kernel; d <= 64 and M <= 16 (checked by the API layer).
hipError_t launch_dp1d(const float *X, const float *W, const float *bias, float inv_lengthscale, int64_t N,
                       int64_t L, int d, int M, int F, float *out, int64_t ld_out, hipStream_t stream);

// RFSF-TRP second stage: recurrence over time on the projected increments P[n_seq*L][M][Q]; M <= 16.
hipError_t launch_trp_scan(const float *P, int64_t n_seq, int64_t L, int M, int Q, float *out, int64_t ld_out,
                           hipStream_t stream);

hipError_t launch_normalize(float *Phi, int64_t N, int64_t ld, int M, int D, hipStream_t stream);

// Benchmark helper (csrc/probe.hip): read, write, non-temporal write, copy GB/s over `scratch`, fp32 matrix and
// fp32 vector TFLOP/s of issue loops, in this order; waits for the stream.
hipError_t probe_peaks(void *scratch, size_t bytes, double out[6], hipStream_t stream);
hipError_t launch_validate_tables(const int32_t *hash, const float *sign, int64_t count, int D,
                                  int *flag, hipStream_t stream);


// Per-kernel event timing (see rfsf_ts_profile_enable). A Scope records a start event when
// constructed and a stop event when destroyed, if profiling is on.
enum KernelClass { kRffIncrements = 0, kSketchFftScan = 1, kGram = 2, kNormalize = 3, kDp1d = 4, kTrpProject = 5, kTrpScan = 6, kNumKernelClasses = 7 };
struct ProfileScope {
    ProfileScope(KernelClass k, hipStream_t stream, bool allowed = true);
    ~ProfileScope();
    int slot;
    hipStream_t stream;
};

}  // namespace rfsf
