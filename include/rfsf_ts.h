/*
 * rfsf_ts.h -- C ABI of the MI355X (gfx950) library for tensor-sketched Random
 * Fourier Signature Features (RFSF-TS, order p = 1) and the linear Gram of the
 * features.
 *
 * Symbols used throughout (the paper's own letters in brackets):
 *   N  sequences                      L  time points per sequence, T = L-1 increments
 *   d  state dimension                M  truncation level
 *   F  random Fourier frequencies per level [paper: D]; the static features have 2F dims
 *   D  count-sketch buckets per level [paper: Q]; powers of two in [2, 4096] and the values 100,
 *      200, 500, 1000 (the projection sizes of the paper's experiments, Sec. 4) have transforms of
 *      exactly that length and are fastest (D < 64 runs in a transform of 64 points); any other D is
 *      accepted as long as M*(D-1)+1 <= 8192 (the convolutions are then evaluated as linear ones with
 *      a longer power-of-two transform and folded modulo D at the end)
 *
 * General rules for every entry point
 *   - Every data pointer is a DEVICE pointer on the current HIP device, owned by
 *     the caller. The library never frees or keeps caller memory and allocates
 *     nothing that the caller sees.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is the
 *     default stream). The calls do not synchronise the device; results are
 *     ready when the stream has drained. (rfsf_ts_features builds its sketch tables
 *     on a stream the library owns, forked from and joined back into `hip_stream`
 *     with events, so the ordering seen by the caller is that of `hip_stream`.)
 *   - Return value: RFSF_OK (0) or a negative RFSF_E_* code. After an argument
 *     error (every code except RFSF_E_HIP) nothing has been enqueued and no output byte
 *     has been written. After RFSF_E_HIP earlier kernels of the call may have been
 *     enqueued; the outputs and the workspace are then unspecified, but nothing of the
 *     library touches them any more once `hip_stream` has drained.
 *   - Threads: the library keeps process-wide state (the side stream and its two events,
 *     the optional profiling record) without locks. Calls from several host threads must
 *     be serialised by the caller; calls from one thread on several streams are fine.
 */
#ifndef RFSF_TS_H
#define RFSF_TS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    RFSF_OK = 0,
    RFSF_E_NULLPTR = -1,            /* a required pointer is NULL                         */
    RFSF_E_BAD_SHAPE = -2,          /* N < 0, L < 1, d < 1, M < 1, F < 1 or size overflow */
    RFSF_E_D_NOT_POW2 = -3,         /* D neither a power of two in [2, 4096] nor small    */
                                    /* enough for the linear route, M*(D-1)+1 <= 8192     */
    RFSF_E_BAD_STRIDE = -4,         /* a leading dimension is smaller than the row        */
    RFSF_E_BAD_LENGTHSCALE = -5,    /* lengthscale is not a finite number > 0             */
    RFSF_E_WORKSPACE_TOO_SMALL = -6,/* workspace cannot hold one chunk (see below)        */
    RFSF_E_HIP = -7,                /* a HIP runtime call or kernel launch failed         */
    RFSF_E_BAD_TABLE = -8,          /* hash outside [0, D) or sign not +-1 (validate)     */
    RFSF_E_UNSUPPORTED = -9,        /* valid but outside what the kernels cover           */
    RFSF_E_STATIC_SCRATCH_TOO_SMALL = -10 /* rfsf_ts_features_static: one sequence needs  */
                                    /* more than the built-in scratch                     */
};

typedef struct {
    int64_t N, L;        /* sequences, time points (L >= 1)                                */
    int32_t d, M, F, D;  /* state dim, levels, frequencies per level, buckets per level    */
    int64_t ld_out;      /* row stride of `out` in floats, >= 1 + M*D                      */
    int32_t rff_bf16;    /* 0: fp32 projection. 1: W rounded to bf16, X split into two     */
                         /* bf16 terms, products accumulated in fp32 on the matrix cores   */
    int32_t order;       /* signature order p: 0 or 1 -> strictly increasing time tuples    */
                         /* (the default); 2, 3 -> a time step may be used up to p times in  */
                         /* a row, q equal indices weighted 1/q! (Sec. 2.1, Sec. 3.5 eq.     */
                         /* (ts_rec), the terms q <= p). 3 needs a power-of-two D in         */
                         /* [64, 2048] (or a transform of that length), M <= 8. Larger: no.  */
} rfsf_ts_shape;

/* Human-readable text for a return code. Never NULL. Host pointer, static storage. */
const char *rfsf_ts_strerror(int code);

/*
 * Scratch memory for rfsf_ts_features.
 *   *recommended_bytes : size at which the whole batch (or a large chunk of it) is
 *                        processed per kernel launch;
 *   *minimum_bytes     : smallest size accepted (one chunk of sequences).
 * Either output pointer may be NULL. The workspace holds the per-call sketch tables and
 * the time increments of the random Fourier features of one chunk of sequences
 * (Sec. 3.2, eq. (rfsf), the factors nabla phi_m) between the two kernels, and, when the
 * sequences are cut in time (rfsf_ts_time_cut), the feature rows of the pieces; its layout is
 * private.
 */
int rfsf_ts_workspace_bytes(const rfsf_ts_shape *shape,
                            size_t *recommended_bytes, size_t *minimum_bytes);

/*
 * How rfsf_ts_features (and _ragged, _static) will cut the sequences of this shape in time. A batch of few
 * long sequences (Sec. 4 measures 10 sequences of up to 1e5 points) cannot fill the GPU with one workgroup
 * per sequence, so each sequence is cut into *pieces pieces of *pairs_per_piece pairs of time steps, the
 * recurrence of Sec. 3.5, eq. (ts_rec) is run on every piece for each first tensor position 1..M, and the
 * pieces are joined with the concatenation identity of iterated sums (the level-m block of x followed by y
 * is the sum over j of the circular convolution of x's level-j block with y's block for positions j+1..m;
 * a product per bin in the transform domain, where the pieces' accumulators are kept) before the final
 * transforms. The result is the same feature map up to fp32 rounding. *pieces = 1 means no cut: more than 64 sequences,
 * sequences too short to give every piece 32 pairs and the batch at least M+1 pieces each,
 * M = 1 or M > 8, or a shape outside the tuned kernels. A function of the shape alone (host code, no GPU
 * work); either output pointer may be NULL. Returns the shape check's code.
 */
int rfsf_ts_time_cut(const rfsf_ts_shape *shape, int32_t *pieces, int64_t *pairs_per_piece);

/*
 * RFSF-TS feature map (Sec. 3.5, eqs. (cs), (ts_def), (ts), (ts_rec), order p = shape->order, on
 * top of the random Fourier features of Sec. 3.1, eq. (rff), one independent map
 * per level as in Sec. 3.2).
 *
 * For each sequence n and level m = 1..M:
 *   theta      = (X[n,t,:] . W[m,:,a]) / lengthscale                a = 0..F-1
 *   phi_m(x_t) = F^{-1/2} (cos theta_0..F-1, sin theta_0..F-1)      2F numbers: cos block first
 *   delta_m[k] = phi_m(x_k) - phi_m(x_{k-1})                        k = 1..T
 *   c_m[k][j]  = sum_{a: hash[m,a] = j} sign[m,a] * delta_m[k][a]   j = 0..D-1
 *   Phi_m      = sum_{k_1 < ... < k_m} c_1[k_1] (*) ... (*) c_m[k_m]   (*) circular convolution mod D
 *                (order 2: sum over k_1 <= ... <= k_m with no index more than twice, each pair of
 *                equal indices weighted 1/2)
 * and out[n, 0] = 1, out[n, 1 + (m-1) D + j] = Phi_m[j].
 *
 *   X     [N, L, d]  float32, row-major, contiguous
 *   W     [M, d, F]  float32 (standard normal draws; the library divides by lengthscale.
 *                    A caller holding pre-scaled frequencies passes lengthscale = 1)
 *   hash  [M, 2F]    int32 in [0, D)      (not checked here: see rfsf_ts_validate_tables;
 *                    out-of-range values are reduced modulo D, never used as addresses)
 *   sign  [M, 2F]    float32 in {+1, -1}  (only the sign bit is used)
 *   out   [N, ld_out] float32; columns 0 .. M*D of every row are written, the rest untouched
 *   workspace, workspace_bytes: scratch from rfsf_ts_workspace_bytes (>= minimum);
 *                    contents on entry are irrelevant, contents on exit are unspecified
 *
 * N = 0 is a successful no-op. L = 1 writes out[n,0] = 1 and zeros. Calls that share a
 * workspace must be ordered on one stream.
 */
int rfsf_ts_features(const rfsf_ts_shape *shape,
                     const float *X, const float *W,
                     const int32_t *hash, const float *sign,
                     float lengthscale,
                     float *out,
                     void *workspace, size_t workspace_bytes,
                     void *hip_stream);

/*
 * rfsf_ts_features for a batch of sequences of different lengths (appendix, ksig.preprocessing: the package
 * takes variable-length input and tabulates it to a common length). X holds N sequences padded to L points
 * each; lengths[n] in [1, L] is the number of points of sequence n that exist, the content of X beyond them
 * is never used for the result. Row n of `out` equals what rfsf_ts_features gives for X[n, 0 .. lengths[n]-1, :]
 * alone (lengths[n] = 1: (1, 0, ..., 0)).
 *   lengths [N] int64 device pointer, or NULL for "all L" (then identical to rfsf_ts_features). Values outside
 *   [1, L] are clamped into it (they are never used as addresses).
 * Everything else as for rfsf_ts_features, including the workspace sizes.
 */
int rfsf_ts_features_ragged(const rfsf_ts_shape *shape,
                            const float *X, const int64_t *lengths, const float *W,
                            const int32_t *hash, const float *sign,
                            float lengthscale,
                            float *out,
                            void *workspace, size_t workspace_bytes,
                            void *hip_stream);

/*
 * rfsf_ts_features for callers that cannot allocate device memory: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments, same results and
 * same error codes as rfsf_ts_features, minus the workspace: the sketch tables and the increments
 * of one chunk of sequences live in a 64 MiB array that is part of the library's code object
 * (one copy per GPU the library runs on, held until the process ends). The call allocates nothing
 * and creates no streams or events: the tables are built on `hip_stream` itself and the optional
 * profiling record is not fed. The batch is processed in as many launches as the 64 MiB allow;
 * a shape whose single sequence (L*M*2F increments plus tables) does not fit returns
 * RFSF_E_STATIC_SCRATCH_TOO_SMALL with nothing enqueued. The first call on a device looks up the
 * array's device address once (make that call outside a graph capture). All calls on one GPU share
 * the array: calls that overlap in time on one GPU (two streams, two threads) race on it; order
 * them on one stream. Contents between calls are unspecified and nothing relies on them.
 */
int rfsf_ts_features_static(const rfsf_ts_shape *shape,
                            const float *X, const float *W,
                            const int32_t *hash, const float *sign,
                            float lengthscale,
                            float *out,
                            void *hip_stream);

/*
 * Opt-in device pass that checks the table contents: every hash[m,a] in [0, D) and every
 * sign[m,a] equal to +1 or -1. Synchronises `hip_stream` (it has to read the result).
 * Returns RFSF_OK or RFSF_E_BAD_TABLE.
 */
int rfsf_ts_validate_tables(const int32_t *hash, const float *sign,
                            int32_t M, int32_t F, int32_t D, void *hip_stream);

/*
 * Linear Gram of primal features (Sec. 1: the Gram matrix of a low-rank feature map is the
 * product of the feature matrix with its transpose; appendix, the feature classes' call operator):
 *   K[i, j] = sum_{c < ncols} PhiX[i, c] * PhiY[j, c]          fp32 in, fp32 accumulate
 *
 *   PhiX [Nx, ldx], PhiY [Ny, ldy]  float32 row-major, ldx, ldy >= ncols (PhiY may equal PhiX)
 *   K    [Nx, ldk]                  float32 row-major, ldk >= Ny; columns 0..Ny-1 written
 *   ncols = 1 + M*D for features made by rfsf_ts_features (the level-0 column is included)
 * Leading dimensions that are multiples of 4 floats with 16-byte aligned bases take the
 * vectorised path; anything else is still correct. Nx = 0 or Ny = 0 is a no-op.
 */
int rfsf_ts_gram(const float *PhiX, int64_t Nx, int64_t ldx,
                 const float *PhiY, int64_t Ny, int64_t ldy,
                 int64_t ncols,
                 float *K, int64_t ldk,
                 void *hip_stream);

/*
 * Level-wise normalisation of feature rows, in place (appendix, class SignatureBase: every
 * signature level is divided by its own norm and the M+1 levels are averaged, so that the
 * normalised kernel 1/(M+1) sum_m k_m(x,y) / sqrt(k_m(x,x) k_m(y,y)) is the plain inner product
 * of the normalised rows and has a unit diagonal):
 *   Phi[n, 0]                 <- Phi[n, 0] / sqrt(M+1)
 *   Phi[n, 1+(m-1)D .. mD]    <- the same block / (its Euclidean norm * sqrt(M+1))
 * A block that is exactly zero (more levels than increments) stays zero.
 *   Phi [N, ld] float32, ld >= 1 + M*D; columns beyond 1 + M*D are untouched. D need not be a
 * power of two here. N = 0 is a no-op.
 */
int rfsf_ts_normalize_features(float *Phi, int64_t N, int64_t ld, int32_t M, int32_t D, void *hip_stream);

/*
 * Sibling variant RFSF-DP-1D (Sec. 3.3, eq. (dp1d), on the one-dimensional random Fourier features
 * of Sec. 3.1, eq. (rff_1d) with the scale of the appendix class RandomFourierFeatures1D): F
 * independent size-1 copies, no sketch and no FFT. For each sequence, level m = 1..M, component i < F:
 *   phi_m(x)[i] = sqrt(2) cos((x . W[m,:,i]) / lengthscale + bias[m,i])
 *   Phi_m[i]    = F^{-1/2} sum_{k_1 < ... < k_m} prod_j (phi_j(x_{k_j})[i] - phi_j(x_{k_j - 1})[i])
 * and out[n, 0] = 1, out[n, 1 + (m-1) F + i] = Phi_m[i]  (1 + M*F columns).
 *   X [N, L, d], W [M, d, F], bias [M, F] (uniform on [0, 2 pi) for an unbiased kernel estimate),
 *   out [N, ld_out], ld_out >= 1 + M*F; all float32 device pointers. No workspace is needed.
 * Limits of this build: d <= 64, M <= 16, d*F*4 < 2^31 (RFSF_E_UNSUPPORTED beyond). N = 0 is a no-op; L = 1 gives
 * (1, 0, ..., 0).
 */
int rfsf_dp1d_features(int64_t N, int64_t L, int32_t d, int32_t M, int32_t F,
                       const float *X, const float *W, const float *bias, float lengthscale,
                       float *out, int64_t ld_out, void *hip_stream);

/*
 * Sibling variant RFSF-TRP (Sec. 3.4, eqs. (trp_def), (trp), (trp_rec); appendix class
 * TensorizedRandomProjection): the feature increments delta_m[k] of rfsf_ts_features (same X, W,
 * lengthscale, cos-then-sin order) are projected per level by an independent Gaussian matrix and
 * combined by Hadamard products instead of circular convolutions:
 *   p_m[k]  = Z[m] delta_m[k]                       Z [M, Q, 2F] float32, i.i.d. N(0,1) draws,
 *                                                   each projection vector contiguous
 *   Phi_m   = Q^{-1/2} sum_{k_1 < ... < k_m} p_1[k_1] (.) ... (.) p_m[k_m]
 * and out[n, 0] = 1, out[n, 1 + (m-1) Q + q] = Phi_m[q]   (1 + M*Q columns).
 * The shape struct is the one of rfsf_ts_features with D meaning Q (any Q >= 1, no power of two
 * needed); ld_out >= 1 + M*Q; rff_bf16 is honoured. M <= 16 in this build. The workspace holds the
 * increments and their projections for one chunk of sequences; sizes from rfsf_trp_workspace_bytes.
 */
int rfsf_trp_workspace_bytes(const rfsf_ts_shape *shape, size_t *recommended_bytes, size_t *minimum_bytes);
int rfsf_trp_features(const rfsf_ts_shape *shape, const float *X, const float *W, const float *Z,
                      float lengthscale, float *out, void *workspace, size_t workspace_bytes,
                      void *hip_stream);

/*
 * Optional per-kernel timing for benchmarks (not part of the method). While enabled, every
 * kernel the library launches is bracketed by HIP events on the stream it is launched on.
 * rfsf_ts_profile_read waits for those events, adds up the elapsed device time per kernel
 * class and the number of launches, and (reset != 0) clears the record. Disabled by default;
 * enabling costs a few microseconds per launch. Process-wide state, not thread-safe.
 */
typedef struct {
    double  ms_rff_increments;   int64_t launches_rff_increments;    /* steps 1-2 kernel */
    double  ms_sketch_fft_scan;  int64_t launches_sketch_fft_scan;   /* steps 3-4 kernel */
    double  ms_gram;             int64_t launches_gram;              /* Gram kernel(s)   */
    double  ms_normalize;        int64_t launches_normalize;         /* normalisation    */
    double  ms_dp1d;             int64_t launches_dp1d;              /* RFSF-DP-1D kernel */
    double  ms_trp_project;      int64_t launches_trp_project;       /* RFSF-TRP GEMMs   */
    double  ms_trp_scan;         int64_t launches_trp_scan;          /* RFSF-TRP scan    */
} rfsf_ts_profile;

int rfsf_ts_profile_enable(int on);
int rfsf_ts_profile_read(rfsf_ts_profile *out, int reset);

/*
 * Benchmark helper (not part of the method): what this GPU gives the simplest kernels of each kind --
 * streaming reads, writes with plain and with non-temporal stores and a copy over `scratch` (device memory,
 * contents destroyed, at least 64 bytes; make it much larger than the 256 MB last-level cache), an issue
 * loop of fp32 matrix instructions (v_mfma_f32_32x32x2f32) and one of fp32 fused multiply-adds. GB/s count
 * bytes read plus bytes written, TFLOP/s two flop per multiply-add. Enqueues on `hip_stream` and waits for
 * it. bench.py prints these beside the published peaks its roofline fractions are quoted against.
 */
typedef struct {
    double read_gbs, write_gbs, write_nt_gbs, copy_gbs;   /* HBM streams */
    double mfma_f32_tflops, valu_f32_tflops;              /* issue loops */
} rfsf_ts_peaks;
int rfsf_ts_probe_peaks(void *scratch, size_t scratch_bytes, rfsf_ts_peaks *out, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RFSF_TS_H */
