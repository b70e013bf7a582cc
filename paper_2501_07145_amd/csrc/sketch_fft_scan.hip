// Steps 3-4 of the RFSF-TS path: CountSketch of every feature increment (Sec. 3.5, eq. (cs)),
// the level recursion over time in the Fourier domain (eq. (ts_rec), second line, p = 1) and
// one inverse transform per level at the end.
//
// With C_m[k] = FFT(CS_m(delta_m[k])) and per-bin accumulators A_m (A_0 = 1), one time step is
//     A_m <- A_m + A_{m-1}(before this step) * C_m[k],   m = 1..M,
// which is the exclusive prefix sum over time of level m-1 times the sketched increment of
// level m, summed over time; Phi_m = IFFT(A_m). Two consecutive time steps share one complex
// FFT (real parts = step k, imaginary parts = step k+1) and are separated again per bin.
#include "rfsf_internal.h"
#include "sketch_fft_scan_tuned.h"
#include "sketch_fft_scan_wide.h"
#include "sketch_fft_scan_dispatch.h"

namespace rfsf {
namespace {

__device__ __forceinline__ float2 cmul(float2 a, float2 b)
{
    return make_float2(fmaf(a.x, b.x, -a.y * b.y), fmaf(a.x, b.y, a.y * b.x));
}
__device__ __forceinline__ float2 cfma(float2 a, float2 b, float2 c)   // a * b + c
{
    return make_float2(fmaf(a.x, b.x, fmaf(-a.y, b.y, c.x)), fmaf(a.x, b.y, fmaf(a.y, b.x, c.y)));
}

// Forward DFT of length D = 2^log2D by radix-2 Stockham passes through two LDS buffers, all
// threads of the workgroup cooperating. tw[t] = exp(-2 pi i t / D), t < D/2. Returns the
// buffer that holds the result in natural order.
__device__ float2 *fft_workgroup(float2 *in, float2 *out, const float2 *tw, int D, int log2D)
{
    for (int s = 0; s < log2D; ++s) {
        const int Ns = 1 << s;
        for (int j = threadIdx.x; j < D / 2; j += blockDim.x) {
            const int k = j & (Ns - 1);
            const float2 w = tw[k << (log2D - 1 - s)];
            const float2 a = in[j];
            const float2 b = cmul(in[j + D / 2], w);
            const int j0 = ((j - k) << 1) + k;
            out[j0] = make_float2(a.x + b.x, a.y + b.y);
            out[j0 + Ns] = make_float2(a.x - b.x, a.y - b.y);
        }
        __syncthreads();
        float2 *t = in; in = out; out = t;
    }
    return in;
}

// float2 elements of the generic kernel's work buffers: two transform buffers, twiddles, the previous level's
// values before each of the two steps (order 2: also level m-2's and the previous level's transforms).
__host__ __device__ constexpr int64_t generic_buffer_elems(int D, int order)
{
    return 2 * (int64_t)D + D / 2 + (order == 2 ? 6 : 2) * (int64_t)(D / 2 + 1);
}

// Generic kernel: any power-of-two transform length D in [2, 8192], any M and F. One workgroup per sequence,
// accumulators in global scratch. Correct everywhere, tuned nowhere.
__global__ __launch_bounds__(256) void sketch_fft_scan_generic(
    const float *__restrict__ dphi, const int32_t *__restrict__ hash, const float *__restrict__ sign,
    int64_t L, const int64_t *__restrict__ lengths, int M, int F, int D, int log2D, int Dout, int order,
    float *__restrict__ out, int64_t ld_out, float2 *__restrict__ state, float2 *__restrict__ scratch)
{
    extern __shared__ float2 sm[];
    const int nb = D / 2 + 1;
    // Work buffers: in LDS when they fit a CU's 160 KB, otherwise (`scratch` not null: transforms of 8192, or
    // of 4096 with order 2) in this sequence's part of the workspace, where they stay L2-resident. The
    // workgroup barriers between the passes make the global writes visible to the whole workgroup.
    float2 *base = scratch ? scratch + (int64_t)blockIdx.x * generic_buffer_elems(D, order) : sm;
    float2 *buf0 = base, *buf1 = base + D, *tw = base + 2 * D;
    float2 *P0 = tw + D / 2, *P1 = P0 + nb;
    float2 *Q0 = P1 + nb, *Q1 = Q0 + nb, *C0p = Q1 + nb, *C1p = C0p + nb;     // order 2 only (allocated then)
    const int64_t n = blockIdx.x;
    // this sequence's own number of points when the batch has variable lengths (clamped to [1, L])
    const int64_t Ln = lengths ? (lengths[n] < 1 ? 1 : (lengths[n] > L ? L : lengths[n])) : L;
    const int64_t T = Ln - 1;
    const int twoF = 2 * F;
    const int64_t rf = (int64_t)M * twoF;
    float2 *A = state + n * M * nb;

    for (int k = threadIdx.x; k < D / 2; k += blockDim.x) {
        float s, c;
        sincospif(2.0f * (float)k / (float)D, &s, &c);
        tw[k] = make_float2(c, -s);
    }
    for (int i = threadIdx.x; i < M * nb; i += blockDim.x) A[i] = make_float2(0.f, 0.f);
    __syncthreads();

    for (int64_t k = 0; k < T; k += 2) {
        const bool two = k + 1 < T;
        const float *row0 = dphi + (n * L + k) * rf;
        const float *row1 = row0 + rf;
        for (int m = 0; m < M; ++m) {
            for (int i = threadIdx.x; i < D; i += blockDim.x) buf0[i] = make_float2(0.f, 0.f);
            __syncthreads();
            for (int a = threadIdx.x; a < twoF; a += blockDim.x) {
                const int h = ((hash[m * twoF + a] % Dout) + Dout) % Dout;      // D > Dout: linear, folded at the end
                const float s = copysignf(1.0f, sign[m * twoF + a]);   // increments arrive halved
                const float v0 = row0[m * twoF + a];
                const float v1 = two ? row1[m * twoF + a] : 0.f;
                atomicAdd(&buf0[h].x, s * v0);
                atomicAdd(&buf0[h].y, s * v1);
            }
            __syncthreads();
            const float2 *Z = fft_workgroup(buf0, buf1, tw, D, log2D);
            for (int f = threadIdx.x; f < nb; f += blockDim.x) {
                const float2 z = Z[f], zc = Z[(D - f) & (D - 1)];
                const float2 C0 = make_float2(z.x + zc.x, z.y - zc.y);
                const float2 C1 = make_float2(z.y + zc.y, zc.x - z.x);
                const float2 p0 = m == 0 ? make_float2(1.f, 0.f) : P0[f];
                const float2 p1 = m == 0 ? make_float2(1.f, 0.f) : P1[f];
                const float2 a_old = A[m * nb + f];
                float2 a_mid = cfma(p0, C0, a_old);
                float2 a_new;
                if (order == 2 && m > 0) {      // + 1/2 A_{m-2}(before the step) C_{m-1} C_m
                    const float2 q0 = m == 1 ? make_float2(1.f, 0.f) : Q0[f];
                    const float2 q1 = m == 1 ? make_float2(1.f, 0.f) : Q1[f];
                    a_mid = cfma(make_float2(0.5f * q0.x, 0.5f * q0.y), cmul(C0p[f], C0), a_mid);
                    a_new = cfma(p1, C1, a_mid);
                    a_new = cfma(make_float2(0.5f * q1.x, 0.5f * q1.y), cmul(C1p[f], C1), a_new);
                } else {
                    a_new = cfma(p1, C1, a_mid);
                }
                if (order == 2) {
                    Q0[f] = p0;
                    Q1[f] = p1;
                    C0p[f] = C0;
                    C1p[f] = C1;
                }
                A[m * nb + f] = a_new;
                P0[f] = a_old;
                P1[f] = a_mid;
            }
            __syncthreads();
        }
    }

    // Phi_m = IFFT(A_m) = Re(FFT(conj(Y))) / D with Y the Hermitian extension of A_m.
    const float invD = 1.0f / (float)D;
    float *row = out + n * ld_out;
    if (threadIdx.x == 0) row[0] = 1.0f;
    for (int m = 0; m < M; ++m) {
        for (int f = threadIdx.x; f < nb; f += blockDim.x) {
            const float2 y = A[m * nb + f];
            buf0[f] = make_float2(y.x, -y.y);
            if (f > 0 && f < D / 2) buf0[D - f] = y;
        }
        __syncthreads();
        const float2 *Z = fft_workgroup(buf0, buf1, tw, D, log2D);
        for (int j = threadIdx.x; j < Dout; j += blockDim.x) {
            float acc = 0.f;
            for (int e = j; e < D; e += Dout) acc += Z[e].x;
            row[1 + (int64_t)m * Dout + j] = acc * invD;
        }
        __syncthreads();
    }
}

// Builds the per-level tables of the tuned kernel (layout: tuned::TableLayout). One workgroup per
// level. rank(a) = number of earlier coordinates of the level in the same bucket; ranks 0 and 1
// go to the gather words, ranks >= 2 become fold entries, ordered by rank and padded so that a
// round of G entries never mixes two ranks (hence never repeats a bucket).
constexpr int kTableThreads = 1024;

__global__ __launch_bounds__(1024) void build_tables_kernel(
    const int32_t *__restrict__ hash, const float *__restrict__ sign, int twoF, int D, int Dout, int G, uint32_t coord_base,
    uint32_t zero_off, uint32_t *__restrict__ table)
{
    extern __shared__ __attribute__((aligned(16))) int table_scratch[];
    const int tf4 = (twoF + 3) & ~3;              // keeps the arrays 16-byte aligned
    int *h = table_scratch, *rk = h + tf4, *cls = rk + tf4, *src0 = cls + tf4 + 4, *src1 = src0 + D;
    __shared__ int max_rank, n_rounds;
    const int m = blockIdx.x, tid = threadIdx.x;
    const tuned::TableLayout tl = tuned::table_layout(D, G, twoF);
    uint32_t *tab = table + (int64_t)m * tl.words;
    (void)sign;                           // applied by the producing kernel

    for (int a = tid; a < twoF; a += kTableThreads) h[a] = ((hash[(int64_t)m * twoF + a] % Dout) + Dout) % Dout;
    for (int e = tid; e < D; e += kTableThreads) { src0[e] = -1; src1[e] = -1; }
    for (int r = tid; r <= twoF; r += kTableThreads) cls[r] = 0;
    if (tid == 0) max_rank = 0;
    __syncthreads();
    for (int a = tid; a < twoF; a += kTableThreads) {
        const int ha = h[a];
        int r = 0, a2 = 0;
        for (; a2 + 8 <= a; a2 += 8) {              // wide LDS reads keep the loop off the LDS latency
            const int4 u = *reinterpret_cast<const int4 *>(h + a2), w = *reinterpret_cast<const int4 *>(h + a2 + 4);
            r += (u.x == ha) + (u.y == ha) + (u.z == ha) + (u.w == ha) + (w.x == ha) + (w.y == ha) + (w.z == ha) + (w.w == ha);
        }
        for (; a2 < a; ++a2) r += h[a2] == ha;
        rk[a] = r;
        if (r == 0) src0[h[a]] = a;
        else if (r == 1) src1[h[a]] = a;
        else { atomicAdd(&cls[r], 1); atomicMax(&max_rank, r); }
    }
    __syncthreads();
    if (tid == 0) {                       // class sizes -> start offsets, each class padded to G
        int off = 0;
        for (int r = 2; r <= max_rank; ++r) {
            const int c = cls[r];
            cls[r] = off;
            off += (c + G - 1) / G * G;
        }
        n_rounds = off / G;
        tab[0] = (uint32_t)n_rounds;
    }
    __syncthreads();
    for (int i = tid; i < n_rounds * G; i += kTableThreads) tab[tl.fold + i] = zero_off | (tuned::kFoldPad << 16);
    for (int e = tid; e < D; e += kTableThreads) {
        const uint32_t s0 = src0[e] >= 0 ? coord_base + (uint32_t)src0[e] * 8u : zero_off;
        const uint32_t s1 = src1[e] >= 0 ? coord_base + (uint32_t)src1[e] * 8u : zero_off;
        tab[tl.gather + e] = s0 | (s1 << 16);
    }
    __syncthreads();                      // padding entries are in place before the real ones land
    for (int a = tid; a < twoF; a += kTableThreads) {
        const int r = rk[a];
        if (r < 2) continue;
        int idx = 0, a2 = 0;
        for (; a2 + 8 <= a; a2 += 8) {
            const int4 u = *reinterpret_cast<const int4 *>(rk + a2), w = *reinterpret_cast<const int4 *>(rk + a2 + 4);
            idx += (u.x == r) + (u.y == r) + (u.z == r) + (u.w == r) + (w.x == r) + (w.y == r) + (w.z == r) + (w.w == r);
        }
        for (; a2 < a; ++a2) idx += rk[a2] == r;
        tab[tl.fold + cls[r] + idx] = (coord_base + (uint32_t)a * 8u) | ((coord_base + (uint32_t)src0[h[a]] * 8u) << 16);
    }
}

__global__ void fill_trivial_kernel(float *out, int64_t n_seq, int64_t ld_out, int64_t ncols)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_seq * ncols) return;
    const int64_t n = i / ncols, c = i % ncols;
    out[n * ld_out + c] = c == 0 ? 1.0f : 0.0f;
}

__global__ void validate_tables_kernel(const int32_t *hash, const float *sign, int64_t count, int D, int *flag)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    const bool ok = hash[i] >= 0 && hash[i] < D && (sign[i] == 1.0f || sign[i] == -1.0f);
    if (!ok) atomicOr(flag, 1);
}

}  // namespace

namespace {
using tuned::kLdsPerCu;
size_t generic_lds_bytes(int D, int order) { return sizeof(float2) * (size_t)generic_buffer_elems(D, order); }
bool generic_in_global(int D, int order) { return generic_lds_bytes(D, order) > kLdsPerCu; }
}  // namespace

size_t sketch_fft_scan_state_bytes(int64_t n_seq, int M, int D, int order)
{
    size_t per = (size_t)M * (size_t)(D / 2 + 1) * sizeof(float2);
    if (generic_in_global(D, order)) per += generic_lds_bytes(D, order);     // work buffers behind the accumulators
    return (size_t)n_seq * per;
}

namespace {
struct TunedGeometry { int G /* entries per fold round */, PD, FPW, NTWL; };
// transforms of 4096 and 8192: the kernel of sketch_fft_scan_wide.h
bool wide_shape(int D) { return D == 4096 || D == 8192; }
size_t table_builder_lds(int twoF, int D) { return sizeof(int) * (size_t)(3 * ((twoF + 3) & ~3) + 4 + 2 * D); }
bool tuned_geometry(int D, TunedGeometry *g)
{
    if (wide_shape(D)) {
        *g = {64, 0, 1, tuned::Plan<10>::NTWL};
        return true;
    }
    switch (D) {
#define RFSF_GEOM(L2) case 1 << L2: *g = {tuned::Plan<L2>::GF, tuned::Plan<L2>::PD, tuned::Plan<L2>::FPW, tuned::Plan<L2>::NTWL}; return true;
        RFSF_GEOM(6) RFSF_GEOM(7) RFSF_GEOM(8) RFSF_GEOM(9) RFSF_GEOM(10)
#undef RFSF_GEOM
#define RFSF_GEOM(DD) case DD: *g = {tuned::Plan<DD>::GF, tuned::Plan<DD>::PD, tuned::Plan<DD>::FPW, tuned::Plan<DD>::NTWL}; return true;
        RFSF_GEOM(100) RFSF_GEOM(200) RFSF_GEOM(500) RFSF_GEOM(1000)        // exact transforms, 2^a 5^b points
        RFSF_GEOM(2048)                                                     // 32 points per lane
#undef RFSF_GEOM
        default: return false;
    }
}
}  // namespace

size_t sketch_fft_scan_lds_bytes(int M, int F, int D)
{
    TunedGeometry g;
    if (!tuned_geometry(D, &g)) return 0;
    if (wide_shape(D)) return tuned::wide_lds_bytes(D / 1024, M, F);
    int log2d = 0;                        // the key of the kernel's plan: log2 D, or D itself for the exact lengths
    while ((1 << log2d) < D) ++log2d;
    if ((1 << log2d) != D || D == 2048) log2d = D;       // (2048 has a plan of its own kind, too)
    // eight wavefronts taking the items in order where the plan prefers that and the slots fit, else one per level
    const size_t preferred = tuned::tuned_lds_bytes(tuned::transforms_in_flight(M, log2d), g.FPW, g.PD, g.NTWL, F);
    return preferred <= kLdsPerCu ? preferred : tuned::tuned_lds_bytes(M, g.FPW, g.PD, g.NTWL, F);
}

bool sketch_fft_scan_is_tuned(int M, int F, int D)
{
    TunedGeometry g;
    // F <= 4032: the staging area (2F rounded up to 128 coordinates) and the zero float2 behind it are
    // addressed with 16-bit byte offsets
    if (M > 8 || F > 4032 || !tuned_geometry(D, &g)) return false;
    if (wide_shape(D) && table_builder_lds(2 * F, D) > kLdsPerCu) return false;
    return sketch_fft_scan_lds_bytes(M, F, D) <= kLdsPerCu;
}

bool sketch_fft_scan_fits(int M, int F, int D, int order)
{
    return sketch_fft_scan_is_tuned(M, F, D) || order <= 2;
}

size_t sketch_fft_scan_table_bytes(int M, int F, int D)
{
    TunedGeometry g;
    if (!sketch_fft_scan_is_tuned(M, F, D) || !tuned_geometry(D, &g)) return 0;
    return sizeof(uint32_t) * (size_t)M * tuned::table_layout(D, g.G, 2 * F).words;
}

hipError_t launch_pack_tables(const int32_t *hash, const float *sign, int M, int F, int D, int Dout,
                              uint32_t *table, hipStream_t stream)
{
    TunedGeometry g;
    if (!sketch_fft_scan_is_tuned(M, F, D) || !tuned_geometry(D, &g)) return hipSuccess;   // generic kernel: no table
    const int twoF = 2 * F;
    const size_t lds = table_builder_lds(twoF, D);
    if (lds > 64 * 1024) {
        static size_t granted = 0;
        if (lds > granted) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(build_tables_kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            granted = lds;
        }
    }
    // byte offsets within a slot: of coordinate 0 and of the float2 that is always zero
    const uint32_t coord_base = wide_shape(D) ? 8u * tuned::kWideStageBase : 0u;
    const uint32_t zero_off = wide_shape(D) ? 0u : 8u * (uint32_t)tuned::zero_slot(g.PD, twoF);
    hipLaunchKernelGGL(build_tables_kernel, dim3((unsigned)M), dim3(kTableThreads), lds, stream, hash, sign, twoF, D, Dout,
                       g.G, coord_base, zero_off, table);
    return hipGetLastError();
}

hipError_t launch_sketch_fft_scan(const float *dphi, const int32_t *hash, const float *sign,
                                  const uint32_t *table, int64_t n_seq, int64_t L, const int64_t *lengths, int M, int F,
                                  int D, int Dout, int order, float *out, int64_t ld_out, float *state,
                                  hipStream_t stream, TimeCut cut)
{
    if (n_seq == 0) return hipSuccess;
    if (cut.pieces < 1 || cut.pairs < 1 || cut.row_levels < M || n_seq * cut.pieces > 0x7fffffffLL) return hipErrorInvalidValue;
    int log2D = 0;
    while ((1 << log2D) < D) ++log2D;
    if (sketch_fft_scan_is_tuned(M, F, D)) {
        switch (D) {
            case 100: return tuned::dispatch_levels_100(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 200: return tuned::dispatch_levels_200(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 500: return tuned::dispatch_levels_500(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 1000: return tuned::dispatch_levels_1000(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 2048: return tuned::dispatch_levels_2048(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            default: break;
        }
        switch (log2D) {
            case 6: return tuned::dispatch_levels_6(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 7: return tuned::dispatch_levels_7(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 8: return tuned::dispatch_levels_8(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 9: return tuned::dispatch_levels_9(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 10: return tuned::dispatch_levels_10(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 12: return tuned::dispatch_levels_12(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            case 13: return tuned::dispatch_levels_13(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
            default: return hipErrorInvalidValue;
        }
    }
    if (order > 2) return hipErrorInvalidValue;           // order 3 exists in the tuned kernel only
    if (cut.pieces != 1 || cut.row_levels != M || cut.mode != 0) return hipErrorInvalidValue;      // and so do cuts in time
    const bool in_global = generic_in_global(D, order);
    const size_t lds = in_global ? 0 : generic_lds_bytes(D, order);
    static size_t lds_granted = 0;        // per process; raising the limit is idempotent
    if (lds > 64 * 1024 && lds > lds_granted) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(sketch_fft_scan_generic),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        lds_granted = lds;
    }
    float2 *acc = reinterpret_cast<float2 *>(state);
    float2 *scratch = in_global ? acc + n_seq * M * (D / 2 + 1) : nullptr;
    hipLaunchKernelGGL(sketch_fft_scan_generic, dim3((unsigned)n_seq), dim3(256), lds, stream,
                       dphi, hash, sign, L, lengths, M, F, D, log2D, Dout, order, out, ld_out, acc, scratch);
    return hipGetLastError();
}

hipError_t launch_fill_trivial(float *out, int64_t n_seq, int64_t ld_out, int64_t ncols, hipStream_t stream)
{
    const int64_t total = n_seq * ncols;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_trivial_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       out, n_seq, ld_out, ncols);
    return hipGetLastError();
}

hipError_t launch_validate_tables(const int32_t *hash, const float *sign, int64_t count, int D,
                                  int *flag, hipStream_t stream)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(validate_tables_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream,
                       hash, sign, count, D, flag);
    return hipGetLastError();
}

}  // namespace rfsf
