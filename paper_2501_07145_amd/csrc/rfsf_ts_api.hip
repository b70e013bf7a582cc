// C ABI of librfsf_ts: argument checks, chunking over sequences, kernel launches.
#include "../../include/rfsf_ts.h"
#include "rfsf_internal.h"

#include <cmath>
#include <vector>

namespace rfsf {
namespace {
struct TimedLaunch { hipEvent_t start, stop; KernelClass k; };
bool g_profile_on = false;
std::vector<TimedLaunch> g_launches;
}  // namespace

ProfileScope::ProfileScope(KernelClass k, hipStream_t s, bool allowed) : slot(-1), stream(s)
{
    if (!g_profile_on || !allowed) return;
    TimedLaunch t{nullptr, nullptr, k};
    if (hipEventCreate(&t.start) != hipSuccess) return;
    if (hipEventCreate(&t.stop) != hipSuccess) { (void)hipEventDestroy(t.start); return; }
    (void)hipEventRecord(t.start, stream);
    g_launches.push_back(t);
    slot = (int)g_launches.size() - 1;
}
ProfileScope::~ProfileScope()
{
    if (slot >= 0) (void)hipEventRecord(g_launches[slot].stop, stream);
}
}  // namespace rfsf

namespace {

constexpr size_t kAlign = 256;
// Increments held per launch, at most. Measured on the N = 10000, L = 200, M = 5, F = 512 batch (41 GB of
// increments): one launch 22.9 ms, two 23.5, four 24.6, sixteen 26.5, 64 launches of 0.64 GB 45 ms; a chunk
// small enough for the last-level cache (64 sequences) cannot fill the chip, since the consumer runs one
// workgroup per sequence. Hence: as few launches as a 48 GiB scratch allows.
constexpr size_t kChunkBytesTarget = (size_t)48 << 30;
constexpr size_t kIncrementTail = 4096;   // the sketch kernel may read up to 1023 floats past the last row

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

bool is_pow2_in_range(int32_t D) { return D >= 2 && D <= 4096 && (D & (D - 1)) == 0; }

// Length of the FFTs. The convolutions are circular modulo D; a transform of P points gives them exactly when
// D divides P (the result, circular modulo P, is folded modulo D at the end) or when P holds the linear
// convolution of M sketches of length D without wrap-around, M*(D-1)+1 numbers. Candidates, in this order: D
// itself when it is a power of two in [2, 4096] or one of 100, 200, 500, 1000 (the bucket counts of the paper's
// own experiments, which have transforms of their own with radices 10, 5, 2); then the powers of two from 64 on
// that are multiples of D or hold the linear convolution. The first one whose shape fits a tuned kernel is
// taken (a small D with many random features, for instance, does not fit at its own length: its wavefronts
// would carry 16 staging areas each); if none does, the first candidate at all, for the generic kernel.
// 0 if there is no candidate up to 8192 points.
int transform_length(int32_t M, int32_t F, int32_t D)
{
    if (D < 1 || D > 4096) return 0;
    const bool pow2 = is_pow2_in_range(D);
    const bool own = pow2 || D == 100 || D == 200 || D == 500 || D == 1000;
    if (own && rfsf::sketch_fft_scan_is_tuned(M, F, D)) return D;
    const int64_t need = (int64_t)M * (D - 1) + 1;
    int first = pow2 ? D : 0;
    for (int64_t P = 2; P <= 8192; P *= 2) {
        if (!(pow2 ? P >= D : P >= need)) continue;
        if (first == 0) first = (int)P;
        if (P >= 64 && rfsf::sketch_fft_scan_is_tuned(M, F, (int)P)) return (int)P;
    }
    return first;
}

int check_shape(const rfsf_ts_shape *s)
{
    if (!s) return RFSF_E_NULLPTR;
    if (s->N < 0 || s->L < 1 || s->d < 1 || s->M < 1 || s->F < 1) return RFSF_E_BAD_SHAPE;
    if (s->N > ((int64_t)1 << 40) || s->L > ((int64_t)1 << 40) || s->d > (1 << 20) || s->M > (1 << 10) ||
        s->F > (1 << 24))
        return RFSF_E_BAD_SHAPE;
    if (transform_length(s->M, s->F, s->D) == 0) return RFSF_E_D_NOT_POW2;
    if (s->order < 0) return RFSF_E_BAD_SHAPE;
    if (s->ld_out < 1 + (int64_t)s->M * s->D) return RFSF_E_BAD_STRIDE;
    return RFSF_OK;
}

// Few long sequences (the shape of the paper's sequence-length runs, Sec. 4: N = 10, L up to 1e5) would keep one
// workgroup per sequence busy and the rest of the chip idle. They are cut in time instead: `pieces` pieces of
// `pairs` pairs of steps per sequence, the sketch kernel launched on every piece once per first tensor
// position (M launches with M, M-1, .. 1 levels: (M+1)/2 times the work), the pieces joined by
// csrc/join_pieces.hip and turned into features by one more launch. A function of the shape alone, so that
// every entry point and every workspace size computes the same sums in the same order. The tuned kernels only
// (any signature order they have: a step's truncated exponential is a factor of the product over steps either way). Measured (M = 5; D = 100, 256, 1024; L = 1e3, 1e4): up to 64 sequences every cut
// into about 1024 / N pieces of at least 32 pairs wins (1.3x at N = 64 .. 30x at N = 1), around 100 sequences
// it is a draw, from 128 on it loses; no cut unless it brings at least M + 1 pieces; at most 128 pieces (they
// are joined one after the other).
struct TimeCutPlan { int pieces; int64_t pairs; };
TimeCutPlan time_cut_plan(const rfsf_ts_shape *s)
{
    const int64_t all_pairs = s->L / 2;                     // L - 1 steps
    const TimeCutPlan whole = {1, (s->L + 1) / 2};
    const int P = transform_length(s->M, s->F, s->D);
    if (s->order > 3 || s->M < 2 || s->M > rfsf::kMaxCutLevels || s->N < 1 || s->N > 64 ||
        !rfsf::sketch_fft_scan_is_tuned(s->M, s->F, P))
        return whole;
    int64_t want = 1024 / s->N;                             // about four workgroups per CU
    if (want > all_pairs / 32) want = all_pairs / 32;
    if (want > 128) want = 128;
    if (want < s->M + 1) return whole;
    for (int levels = 1; levels < s->M; ++levels)           // every launch of the series runs a tuned kernel
        if (!rfsf::sketch_fft_scan_is_tuned(levels, s->F, P)) return whole;
    const int64_t pairs = (all_pairs + want - 1) / want;
    return {(int)((all_pairs + pairs - 1) / pairs), pairs};
}
// floats of one sequence's pieces: per piece and first position a the accumulators of levels a+1 .. M (bins
// 0 .. P/2 of the transform, complex), plus the joined accumulators of the sequence
size_t piece_floats(const rfsf_ts_shape *s, int pieces)
{
    const size_t bins = (size_t)transform_length(s->M, s->F, s->D) / 2 + 1;
    size_t per_piece = 0;
    for (int a = 0; a < s->M; ++a) per_piece += (size_t)(s->M - a) * bins * 2;
    return per_piece * (size_t)pieces + (size_t)s->M * bins * 2;
}

// Bytes of workspace one sequence needs: its increment rows plus its state (the generic kernel's
// accumulators; the rows of its pieces when the sequences are cut in time).
void per_sequence_bytes(const rfsf_ts_shape *s, size_t *incr, size_t *state)
{
    // rows of increments per sequence: L in the row layout, L rounded up to even in the pair layout
    *incr = (size_t)((s->L + 1) & ~(int64_t)1) * (size_t)s->M * 2u * (size_t)s->F * sizeof(float);
    *state = rfsf::sketch_fft_scan_state_bytes(1, s->M, transform_length(s->M, s->F, s->D), s->order == 2 ? 2 : 1);
    const TimeCutPlan plan = time_cut_plan(s);
    if (plan.pieces > 1) *state += sizeof(float) * piece_floats(s, plan.pieces);
}

// Fixed part: packed hash/sign table plus room for aligning the three sections.
size_t fixed_bytes(const rfsf_ts_shape *s)
{
    return align_up(rfsf::sketch_fft_scan_table_bytes(s->M, s->F, transform_length(s->M, s->F, s->D))) + kIncrementTail +
           3 * kAlign;
}

int64_t chunk_for(const rfsf_ts_shape *s, size_t bytes)
{
    size_t incr, state;
    per_sequence_bytes(s, &incr, &state);
    const size_t fixed = fixed_bytes(s);
    if (bytes < fixed) return 0;
    return (int64_t)((bytes - fixed) / (incr + state));
}

// The sketch tables depend only on hash/sign, not on the increments, so they are built on a side
// stream (default priority) while the first projection kernel runs. The side stream first waits for
// everything already enqueued on the caller's stream (an earlier call may still be reading the
// tables), and the caller's stream waits for the tables before the first sketch kernel.
// Process-wide, created on first use; if anything fails the build simply runs on the caller's stream.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t begin = nullptr, done = nullptr;
    int device = -1;            // the device the stream and events belong to
    bool usable = false;
};
SideStream &side_stream()
{
    static SideStream s;
    static bool tried = false;
    if (!tried) {
        tried = true;
        s.usable = hipGetDevice(&s.device) == hipSuccess &&
                   hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) == hipSuccess &&
                   hipEventCreateWithFlags(&s.begin, hipEventDisableTiming) == hipSuccess &&
                   hipEventCreateWithFlags(&s.done, hipEventDisableTiming) == hipSuccess;
    }
    return s;
}
bool side_stream_matches_current_device(const SideStream &s)
{
    int dev = -1;
    return s.usable && hipGetDevice(&dev) == hipSuccess && dev == s.device;
}

}  // namespace

extern "C" const char *rfsf_ts_strerror(int code)
{
    switch (code) {
        case RFSF_OK: return "success";
        case RFSF_E_NULLPTR: return "a required pointer is NULL";
        case RFSF_E_BAD_SHAPE: return "bad shape: need N >= 0, L >= 1, d >= 1, M >= 1, F >= 1 within limits";
        case RFSF_E_D_NOT_POW2: return "D must be a power of two in [2, 4096], or satisfy M*(D-1)+1 <= 8192";
        case RFSF_E_BAD_STRIDE: return "leading dimension smaller than the row length";
        case RFSF_E_BAD_LENGTHSCALE: return "lengthscale must be finite and > 0";
        case RFSF_E_WORKSPACE_TOO_SMALL: return "workspace smaller than rfsf_ts_workspace_bytes' minimum";
        case RFSF_E_HIP: return "HIP runtime error";
        case RFSF_E_BAD_TABLE: return "hash outside [0, D) or sign not +-1";
        case RFSF_E_UNSUPPORTED: return "configuration not supported by this build";
        case RFSF_E_STATIC_SCRATCH_TOO_SMALL:
            return "one sequence needs more than the 64 MiB built-in scratch: use rfsf_ts_features with a workspace";
        default: return "unknown rfsf_ts error code";
    }
}

extern "C" int rfsf_ts_workspace_bytes(const rfsf_ts_shape *shape, size_t *recommended_bytes,
                                       size_t *minimum_bytes)
{
    const int rc = check_shape(shape);
    if (rc != RFSF_OK) return rc;
    size_t incr, state;
    per_sequence_bytes(shape, &incr, &state);
    const size_t per = incr + state;
    int64_t chunk = (int64_t)(kChunkBytesTarget / per);
    if (chunk < 1) chunk = 1;
    if (chunk > shape->N) chunk = shape->N > 0 ? shape->N : 1;
    // equal-sized chunks: no small trailing launch
    if (shape->N > 0) {
        const int64_t nchunks = (shape->N + chunk - 1) / chunk;
        chunk = (shape->N + nchunks - 1) / nchunks;
    }
    if (recommended_bytes) *recommended_bytes = (size_t)chunk * per + fixed_bytes(shape);
    if (minimum_bytes) *minimum_bytes = per + fixed_bytes(shape);
    return RFSF_OK;
}

extern "C" int rfsf_ts_time_cut(const rfsf_ts_shape *shape, int32_t *pieces, int64_t *pairs_per_piece)
{
    const int rc = check_shape(shape);
    if (rc != RFSF_OK) return rc;
    const TimeCutPlan plan = time_cut_plan(shape);
    if (pieces) *pieces = plan.pieces;
    if (pairs_per_piece) *pairs_per_piece = plan.pairs;
    return RFSF_OK;
}

namespace {
// Body of rfsf_ts_features. `may_create` = false keeps the call free of anything that creates runtime
// objects: the tables are then built on the caller's stream (no library-owned stream or events) and no
// profiling events are recorded.
int features_impl(const rfsf_ts_shape *shape, const float *X, const int64_t *lengths, const float *W,
                  const int32_t *hash, const float *sign, float lengthscale, float *out, void *workspace,
                  size_t workspace_bytes, void *hip_stream, bool may_create)
{
    int rc = check_shape(shape);
    if (rc != RFSF_OK) return rc;
    if (!(lengthscale > 0.0f) || !std::isfinite(lengthscale)) return RFSF_E_BAD_LENGTHSCALE;
    if (shape->N == 0) return RFSF_OK;
    if (!X || !W || !hash || !sign || !out) return RFSF_E_NULLPTR;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t ncols = 1 + (int64_t)shape->M * shape->D;

    if (shape->L == 1) {      // no increments: empty sums
        return rfsf::launch_fill_trivial(out, shape->N, shape->ld_out, ncols, stream) == hipSuccess
                   ? RFSF_OK : RFSF_E_HIP;
    }
    if ((int64_t)shape->M * ((shape->F + 127) / 128) > 65535) return RFSF_E_UNSUPPORTED;   // grid limits
    if (shape->rff_bf16 != 0 && shape->d > 128) return RFSF_E_UNSUPPORTED;
    if (shape->order > 3) return RFSF_E_UNSUPPORTED;
    if ((int64_t)shape->M * 2 * shape->F > ((int64_t)1 << 26)) return RFSF_E_UNSUPPORTED;   // 32-bit row offsets
    if (!rfsf::sketch_fft_scan_fits(shape->M, shape->F, transform_length(shape->M, shape->F, shape->D), shape->order < 2 ? 1 : shape->order))
        return RFSF_E_UNSUPPORTED;        // order 3 outside the tuned kernel's shapes
    if (!workspace) return RFSF_E_NULLPTR;
    int64_t chunk = chunk_for(shape, workspace_bytes);
    if (chunk < 1) return RFSF_E_WORKSPACE_TOO_SMALL;
    if (chunk > shape->N) chunk = shape->N;

    size_t incr, state_b;
    per_sequence_bytes(shape, &incr, &state_b);
    char *base = static_cast<char *>(workspace);
    const size_t mis = (size_t)(reinterpret_cast<uintptr_t>(base) % kAlign);
    char *p_table = base + (mis ? kAlign - mis : 0);
    const int P = transform_length(shape->M, shape->F, shape->D);
    char *p_incr = p_table + align_up(rfsf::sketch_fft_scan_table_bytes(shape->M, shape->F, P));
    char *p_state = p_incr + align_up((size_t)chunk * incr + kIncrementTail);
    float *dphi = reinterpret_cast<float *>(p_incr);
    float *state = reinterpret_cast<float *>(p_state);
    uint32_t *table = reinterpret_cast<uint32_t *>(p_table);
    static SideStream no_side;
    SideStream &side = may_create ? side_stream() : no_side;
    bool tables_on_side = false;
    // Error return after the fork: the caller's stream first waits for whatever the side stream still does
    // (the table build writes the workspace), so that the workspace is quiet once `stream` has drained.
    auto fail = [&]() {
        if (tables_on_side) {
            if (hipStreamWaitEvent(stream, side.done, 0) != hipSuccess) (void)hipStreamSynchronize(side.stream);
        }
        return RFSF_E_HIP;
    };
    if (side_stream_matches_current_device(side) && hipEventRecord(side.begin, stream) == hipSuccess &&
        hipStreamWaitEvent(side.stream, side.begin, 0) == hipSuccess) {
        const hipError_t e = rfsf::launch_pack_tables(hash, sign, shape->M, shape->F, P, shape->D, table, side.stream);
        if (hipEventRecord(side.done, side.stream) != hipSuccess) {
            (void)hipStreamSynchronize(side.stream);
            return RFSF_E_HIP;
        }
        tables_on_side = true;
        if (e != hipSuccess) return fail();
    } else if (rfsf::launch_pack_tables(hash, sign, shape->M, shape->F, P, shape->D, table, stream) != hipSuccess) {
        return RFSF_E_HIP;
    }

    const float inv_ls = 1.0f / lengthscale;
    const TimeCutPlan plan = time_cut_plan(shape);
    // the tuned consumer takes the increments in the pair layout with the signs applied, the generic one in
    // the row layout without
    const float *producer_sign = rfsf::sketch_fft_scan_is_tuned(shape->M, shape->F, P) ? sign : nullptr;
    for (int64_t n0 = 0; n0 < shape->N; n0 += chunk) {
        const int64_t cnt = shape->N - n0 < chunk ? shape->N - n0 : chunk;
        {
            rfsf::ProfileScope scope(rfsf::kRffIncrements, stream, may_create);
            if (rfsf::launch_rff_increments(X + n0 * shape->L * shape->d, W, producer_sign, inv_ls, cnt, shape->L, shape->d,
                                            shape->M, shape->F, shape->rff_bf16 != 0, dphi, stream) != hipSuccess)
                return fail();
        }
        if (tables_on_side) {           // join: the tables are needed from here on
            if (hipStreamWaitEvent(stream, side.done, 0) != hipSuccess) return fail();
            tables_on_side = false;
        }
        const int64_t *chunk_lengths = lengths ? lengths + n0 : nullptr;
        if (plan.pieces == 1) {
            rfsf::ProfileScope scope(rfsf::kSketchFftScan, stream, may_create);
            if (rfsf::launch_sketch_fft_scan(dphi, hash, sign, table, cnt, shape->L, chunk_lengths,
                                             shape->M, shape->F, P, shape->D, shape->order < 2 ? 1 : shape->order,
                                             out + n0 * shape->ld_out, shape->ld_out, state, stream,
                                             rfsf::TimeCut::whole(shape->L, shape->M)) != hipSuccess)
                return RFSF_E_HIP;
        } else {
            // sequences cut in time: the accumulators of levels a+1 .. M of every piece for a = 0 .. M-1, the join,
            // and the final transforms of the joined accumulators (timed as one launch of the sketch kernel class)
            rfsf::ProfileScope scope(rfsf::kSketchFftScan, stream, may_create);
            rfsf::PieceRows rows = {};
            const int order = shape->order < 2 ? 1 : shape->order;
            float2 *next = reinterpret_cast<float2 *>(state);
            const size_t bins = (size_t)P / 2 + 1;
            const size_t level_words = rfsf::sketch_fft_scan_table_bytes(shape->M, shape->F, P) / sizeof(uint32_t) / (size_t)shape->M;
            for (int a = 0; a < shape->M; ++a) {
                const int levels = shape->M - a;
                rows.rows[a] = next;
                if (rfsf::launch_sketch_fft_scan(dphi + (size_t)a * 4 * shape->F, hash, sign, table + (size_t)a * level_words,
                                                 cnt, shape->L, chunk_lengths, levels, shape->F, P, shape->D, order,
                                                 out + n0 * shape->ld_out, shape->ld_out, nullptr, stream,
                                                 rfsf::TimeCut{plan.pieces, shape->M, plan.pairs, next, 1}) != hipSuccess)
                    return RFSF_E_HIP;
                next += (size_t)cnt * plan.pieces * levels * bins;
            }
            if (rfsf::launch_join_pieces(rows, cnt, plan.pieces, shape->M, (int)bins, next, stream) != hipSuccess)
                return RFSF_E_HIP;
            if (rfsf::launch_sketch_fft_scan(dphi, hash, sign, table, cnt, shape->L, chunk_lengths, shape->M, shape->F, P,
                                             shape->D, order, out + n0 * shape->ld_out, shape->ld_out, nullptr, stream,
                                             rfsf::TimeCut{1, shape->M, (shape->L + 1) / 2, next, 2}) != hipSuccess)
                return RFSF_E_HIP;
        }
    }
    return RFSF_OK;
}

// Scratch of the entry point that allocates nothing: one array per GPU, part of the library's code object.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
constexpr int kMaxDevices = 64;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
// Device address of `scratch` on the current device, resolved once per device (each GPU holds its own copy
// at its own address); nullptr if the lookup fails.
void *static_scratch_address()
{
    static void *address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    if (!address[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        address[dev] = ptr;
    }
    return address[dev];
}
}  // namespace

extern "C" int rfsf_ts_features(const rfsf_ts_shape *shape, const float *X, const float *W,
                                const int32_t *hash, const float *sign, float lengthscale, float *out,
                                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return features_impl(shape, X, nullptr, W, hash, sign, lengthscale, out, workspace, workspace_bytes, hip_stream,
                         true);
}

extern "C" int rfsf_ts_features_ragged(const rfsf_ts_shape *shape, const float *X, const int64_t *lengths,
                                       const float *W, const int32_t *hash, const float *sign, float lengthscale,
                                       float *out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return features_impl(shape, X, lengths, W, hash, sign, lengthscale, out, workspace, workspace_bytes, hip_stream,
                         true);
}

extern "C" int rfsf_ts_features_static(const rfsf_ts_shape *shape, const float *X, const float *W,
                                       const int32_t *hash, const float *sign, float lengthscale, float *out,
                                       void *hip_stream)
{
    const int rc = check_shape(shape);
    if (rc != RFSF_OK) return rc;
    if (shape->N > 0 && shape->L > 1) {      // one sequence (increments + state) plus the tables must fit
        size_t incr, state;
        per_sequence_bytes(shape, &incr, &state);
        if (incr + state > kStaticScratchBytes || fixed_bytes(shape) > kStaticScratchBytes - (incr + state))
            return RFSF_E_STATIC_SCRATCH_TOO_SMALL;
    }
    void *ptr = static_scratch_address();
    if (!ptr) return RFSF_E_HIP;
    return features_impl(shape, X, nullptr, W, hash, sign, lengthscale, out, ptr, kStaticScratchBytes, hip_stream,
                         false);
}

extern "C" int rfsf_ts_validate_tables(const int32_t *hash, const float *sign, int32_t M, int32_t F,
                                       int32_t D, void *hip_stream)
{
    if (!hash || !sign) return RFSF_E_NULLPTR;
    if (M < 1 || F < 1) return RFSF_E_BAD_SHAPE;
    if (D < 1 || D > 4096) return RFSF_E_D_NOT_POW2;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int *flag = nullptr;
    if (hipMalloc(&flag, sizeof(int)) != hipSuccess) return RFSF_E_HIP;
    int host = 0;
    int rc = RFSF_OK;
    if (hipMemcpyAsync(flag, &host, sizeof(int), hipMemcpyHostToDevice, stream) != hipSuccess ||
        rfsf::launch_validate_tables(hash, sign, (int64_t)M * 2 * F, D, flag, stream) != hipSuccess ||
        hipMemcpyAsync(&host, flag, sizeof(int), hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        rc = RFSF_E_HIP;
    (void)hipFree(flag);
    if (rc != RFSF_OK) return rc;
    return host ? RFSF_E_BAD_TABLE : RFSF_OK;
}

extern "C" int rfsf_ts_gram(const float *PhiX, int64_t Nx, int64_t ldx, const float *PhiY, int64_t Ny,
                            int64_t ldy, int64_t ncols, float *K, int64_t ldk, void *hip_stream)
{
    if (Nx < 0 || Ny < 0 || ncols < 0) return RFSF_E_BAD_SHAPE;
    if (ldx < ncols || ldy < ncols || ldk < Ny) return RFSF_E_BAD_STRIDE;
    if (Nx == 0 || Ny == 0) return RFSF_OK;
    if (!PhiX || !PhiY || !K) return RFSF_E_NULLPTR;
    if ((Nx + 63) / 64 > 65535 || (Ny + 63) / 64 > 2147483647) return RFSF_E_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    rfsf::ProfileScope scope(rfsf::kGram, stream);
    return rfsf::launch_gram(PhiX, Nx, ldx, PhiY, Ny, ldy, ncols, K, ldk, stream) == hipSuccess
               ? RFSF_OK : RFSF_E_HIP;
}

extern "C" int rfsf_ts_normalize_features(float *Phi, int64_t N, int64_t ld, int32_t M, int32_t D,
                                          void *hip_stream)
{
    if (N < 0 || M < 1 || D < 1 || N > 0x7fffffffLL) return RFSF_E_BAD_SHAPE;
    if (ld < 1 + (int64_t)M * D) return RFSF_E_BAD_STRIDE;
    if (N == 0) return RFSF_OK;
    if (!Phi) return RFSF_E_NULLPTR;
    rfsf::ProfileScope scope(rfsf::kNormalize, static_cast<hipStream_t>(hip_stream));
    return rfsf::launch_normalize(Phi, N, ld, M, D, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? RFSF_OK : RFSF_E_HIP;
}

extern "C" int rfsf_dp1d_features(int64_t N, int64_t L, int32_t d, int32_t M, int32_t F, const float *X,
                                  const float *W, const float *bias, float lengthscale, float *out,
                                  int64_t ld_out, void *hip_stream)
{
    if (N < 0 || L < 1 || d < 1 || M < 1 || F < 1 || N > 0x7fffffffLL || L > ((int64_t)1 << 40) || F > (1 << 24))
        return RFSF_E_BAD_SHAPE;
    if (ld_out < 1 + (int64_t)M * F) return RFSF_E_BAD_STRIDE;
    if (!(lengthscale > 0.0f) || !std::isfinite(lengthscale)) return RFSF_E_BAD_LENGTHSCALE;
    if (d > 64 || M > 16 || (F + 255) / 256 > 65535) return RFSF_E_UNSUPPORTED;
    if ((int64_t)d * F * 4 > 0x7fffffffLL) return RFSF_E_UNSUPPORTED;     // a level of W is addressed with 32-bit byte offsets
    if (N == 0) return RFSF_OK;
    if (!X || !W || !bias || !out) return RFSF_E_NULLPTR;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    rfsf::ProfileScope scope(rfsf::kDp1d, stream);
    return rfsf::launch_dp1d(X, W, bias, 1.0f / lengthscale, N, L, d, M, F, out, ld_out, stream) == hipSuccess
               ? RFSF_OK : RFSF_E_HIP;
}

namespace {
int check_trp_shape(const rfsf_ts_shape *s)
{
    if (!s) return RFSF_E_NULLPTR;
    if (s->N < 0 || s->L < 1 || s->d < 1 || s->M < 1 || s->F < 1 || s->D < 1) return RFSF_E_BAD_SHAPE;
    if (s->N > ((int64_t)1 << 40) || s->L >= ((int64_t)1 << 31) || s->d > (1 << 20) || s->F > (1 << 24) ||
        s->D > (1 << 24))
        return RFSF_E_BAD_SHAPE;
    if (s->ld_out < 1 + (int64_t)s->M * s->D) return RFSF_E_BAD_STRIDE;
    if (s->M > 16 || (int64_t)s->M * 2 * s->F > ((int64_t)1 << 26) || (int64_t)s->M * s->D > ((int64_t)1 << 26) ||
        (int64_t)s->M * ((s->F + 127) / 128) > 65535 || (s->rff_bf16 != 0 && s->d > 128))
        return RFSF_E_UNSUPPORTED;
    return RFSF_OK;
}
void trp_per_sequence_bytes(const rfsf_ts_shape *s, size_t *incr, size_t *proj)
{
    *incr = (size_t)s->L * (size_t)s->M * 2u * (size_t)s->F * sizeof(float);
    *proj = (size_t)s->L * (size_t)s->M * (size_t)s->D * sizeof(float);
}
constexpr size_t kTrpFixed = 3 * kAlign;
// Sequences per launch of the TRP kernels: the scan puts the sequence and the per-level GEMMs put 64-row
// tiles of the chunk's L*cnt rows on grid.y, which holds at most 65535.
int64_t trp_chunk_cap(const rfsf_ts_shape *s)
{
    const int64_t by_rows = (int64_t)65535 * 64 / s->L;
    return by_rows < 65535 ? by_rows : 65535;
}
}  // namespace

extern "C" int rfsf_trp_workspace_bytes(const rfsf_ts_shape *shape, size_t *recommended_bytes,
                                        size_t *minimum_bytes)
{
    const int rc = check_trp_shape(shape);
    if (rc != RFSF_OK) return rc;
    size_t incr, proj;
    trp_per_sequence_bytes(shape, &incr, &proj);
    const size_t per = incr + proj;
    if (trp_chunk_cap(shape) < 1) return RFSF_E_UNSUPPORTED;     // one sequence alone exceeds the grid
    int64_t chunk = (int64_t)(kChunkBytesTarget / per);
    if (chunk > trp_chunk_cap(shape)) chunk = trp_chunk_cap(shape);
    if (chunk < 1) chunk = 1;
    if (chunk > shape->N) chunk = shape->N > 0 ? shape->N : 1;
    if (shape->N > 0) {
        const int64_t nchunks = (shape->N + chunk - 1) / chunk;
        chunk = (shape->N + nchunks - 1) / nchunks;
    }
    if (recommended_bytes) *recommended_bytes = (size_t)chunk * per + kTrpFixed;
    if (minimum_bytes) *minimum_bytes = per + kTrpFixed;
    return RFSF_OK;
}

extern "C" int rfsf_trp_features(const rfsf_ts_shape *shape, const float *X, const float *W, const float *Z,
                                 float lengthscale, float *out, void *workspace, size_t workspace_bytes,
                                 void *hip_stream)
{
    int rc = check_trp_shape(shape);
    if (rc != RFSF_OK) return rc;
    if (!(lengthscale > 0.0f) || !std::isfinite(lengthscale)) return RFSF_E_BAD_LENGTHSCALE;
    if (shape->N == 0) return RFSF_OK;
    if (!X || !W || !Z || !out) return RFSF_E_NULLPTR;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int Q = shape->D;
    if (shape->L == 1)
        return rfsf::launch_fill_trivial(out, shape->N, shape->ld_out, 1 + (int64_t)shape->M * Q, stream) == hipSuccess
                   ? RFSF_OK : RFSF_E_HIP;
    if (trp_chunk_cap(shape) < 1) return RFSF_E_UNSUPPORTED;
    if (!workspace) return RFSF_E_NULLPTR;
    size_t incr, proj;
    trp_per_sequence_bytes(shape, &incr, &proj);
    if (workspace_bytes < incr + proj + kTrpFixed) return RFSF_E_WORKSPACE_TOO_SMALL;
    int64_t chunk = (int64_t)((workspace_bytes - kTrpFixed) / (incr + proj));
    if (chunk > shape->N) chunk = shape->N;
    if (chunk > trp_chunk_cap(shape)) chunk = trp_chunk_cap(shape);
    char *base = static_cast<char *>(workspace);
    const size_t mis = (size_t)(reinterpret_cast<uintptr_t>(base) % kAlign);
    float *dphi = reinterpret_cast<float *>(base + (mis ? kAlign - mis : 0));
    float *P = reinterpret_cast<float *>(reinterpret_cast<char *>(dphi) + align_up((size_t)chunk * incr));
    const int twoF = 2 * shape->F;
    const int64_t rf = (int64_t)shape->M * twoF, MQ = (int64_t)shape->M * Q;
    const float inv_ls = 1.0f / lengthscale;
    for (int64_t n0 = 0; n0 < shape->N; n0 += chunk) {
        const int64_t cnt = shape->N - n0 < chunk ? shape->N - n0 : chunk;
        {
            rfsf::ProfileScope scope(rfsf::kRffIncrements, stream);
            if (rfsf::launch_rff_increments(X + n0 * shape->L * shape->d, W, nullptr, inv_ls, cnt, shape->L, shape->d,
                                            shape->M, shape->F, shape->rff_bf16 != 0, dphi, stream) != hipSuccess)
                return RFSF_E_HIP;
        }
        {   // P[:, m, :] = dphi[:, m, :] Z_m^T, one GEMM per level (rows whose increment does not exist are
            // computed too and never read)
            rfsf::ProfileScope scope(rfsf::kTrpProject, stream);
            for (int m = 0; m < shape->M; ++m)
                if (rfsf::launch_gram(dphi + (int64_t)m * twoF, cnt * shape->L, rf, Z + (int64_t)m * Q * twoF, Q, twoF,
                                      twoF, P + (int64_t)m * Q, MQ, stream) != hipSuccess)
                    return RFSF_E_HIP;
        }
        {
            rfsf::ProfileScope scope(rfsf::kTrpScan, stream);
            if (rfsf::launch_trp_scan(P, cnt, shape->L, shape->M, Q, out + n0 * shape->ld_out, shape->ld_out,
                                      stream) != hipSuccess)
                return RFSF_E_HIP;
        }
    }
    return RFSF_OK;
}

extern "C" int rfsf_ts_probe_peaks(void *scratch, size_t scratch_bytes, rfsf_ts_peaks *out, void *hip_stream)
{
    if (!scratch || !out) return RFSF_E_NULLPTR;
    if (scratch_bytes < 64) return RFSF_E_WORKSPACE_TOO_SMALL;
    double v[6];
    if (rfsf::probe_peaks(scratch, scratch_bytes, v, static_cast<hipStream_t>(hip_stream)) != hipSuccess) return RFSF_E_HIP;
    *out = rfsf_ts_peaks{v[0], v[1], v[2], v[3], v[4], v[5]};
    return RFSF_OK;
}

extern "C" int rfsf_ts_profile_enable(int on)
{
    rfsf::g_profile_on = on != 0;
    return RFSF_OK;
}

extern "C" int rfsf_ts_profile_read(rfsf_ts_profile *out, int reset)
{
    if (!out) return RFSF_E_NULLPTR;
    *out = rfsf_ts_profile{0.0, 0, 0.0, 0, 0.0, 0, 0.0, 0, 0.0, 0, 0.0, 0, 0.0, 0};
    int rc = RFSF_OK;
    for (const rfsf::TimedLaunch &t : rfsf::g_launches) {
        float ms = 0.f;
        if (hipEventSynchronize(t.stop) != hipSuccess || hipEventElapsedTime(&ms, t.start, t.stop) != hipSuccess) {
            rc = RFSF_E_HIP;
            continue;
        }
        switch (t.k) {
            case rfsf::kRffIncrements: out->ms_rff_increments += ms; ++out->launches_rff_increments; break;
            case rfsf::kSketchFftScan: out->ms_sketch_fft_scan += ms; ++out->launches_sketch_fft_scan; break;
            case rfsf::kGram: out->ms_gram += ms; ++out->launches_gram; break;
            case rfsf::kNormalize: out->ms_normalize += ms; ++out->launches_normalize; break;
            case rfsf::kDp1d: out->ms_dp1d += ms; ++out->launches_dp1d; break;
            case rfsf::kTrpProject: out->ms_trp_project += ms; ++out->launches_trp_project; break;
            default: out->ms_trp_scan += ms; ++out->launches_trp_scan; break;
        }
    }
    if (reset) {
        for (const rfsf::TimedLaunch &t : rfsf::g_launches) {
            (void)hipEventDestroy(t.start);
            (void)hipEventDestroy(t.stop);
        }
        rfsf::g_launches.clear();
    }
    return rc;
}
