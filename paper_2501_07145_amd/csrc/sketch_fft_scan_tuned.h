// Tuned kernel for steps 3-4 (CountSketch, Fourier-domain level recursion over time, inverse
// transform; Sec. 3.5, eqs. (cs), (ts_def), (ts_rec) with p = 1).
//
// Work decomposition (one workgroup per sequence, M wavefronts, wavefront m owns level m; a transform always
// lives in one wavefront: 16 points per lane up to D = 1024, 32 for D = 2048):
//   per iteration every wavefront handles FPW pairs of consecutive time steps of its level:
//     1. CountSketch as a gather. The signed increments of the 2*FPW time steps arrive in LDS in
//        their natural order (step 2k -> real part, step 2k+1 -> imaginary part of the float2 of
//        coordinate a, one staging area per pair): the producing kernel stores them in exactly this
//        form, signs applied, and they are loaded from global memory straight into LDS
//        (global_load_lds_dwordx4: 16 bytes per lane at LDS base + 16 * lane), without passing
//        through registers and without LDS-write instructions. A table built once per call lists,
//        for every bucket, the first two coordinates that hash to it; the few coordinates that
//        are third or later in their bucket are first folded into the bucket's first coordinate
//        by conflict-free read-add-write rounds (one round per rank, so no two lanes of a round
//        touch the same float2). Then each FFT lane reads the (at most two) sources of each of
//        its R buckets straight into its FFT registers. No LDS atomics (a full-wavefront
//        ds_add_f32 costs ~190 cycles on this chip), no clearing, and the summation order is
//        fixed, so results are bit-reproducible.
//     2. FPW complex FFTs of length D held in the wavefront's LDS slots, G = D/R lanes per
//        transform with R = 16 points per lane in registers (Stockham passes, radix up to 16 in
//        registers, one LDS exchange per pass; no workgroup barrier inside the transform unless it
//        spans two wavefronts),
//   then, after one barrier, every thread owns a few frequency bins, separates the two real
//   transforms of each slot, and advances the accumulators A_1..A_M of its bins by the two
//   time steps (A_m += A_{m-1}(before the step) * C_m, A_0 = 1; with signature order 2 also
//   + 1/2 A_{m-2}(before the step) * C_{m-1} * C_m, with order 3 also + 1/6 A_{m-3} C_{m-2} C_{m-1} C_m:
//   Sec. 3.5 eq. (ts_rec), the terms q = 2, 3).
//   After the last time step, wavefront m transforms A_m back and writes block m of the row.
//   (Fetching the next iteration's rows ahead of time was tried in several placements and was never
//   faster: the pace is set by the instruction streams of the resident workgroups, not by the load
//   latency of one of them. What did pay off every time was more resident wavefronts.)
//
// The increments arrive pre-multiplied by 1/2 and by their CountSketch sign (done by the producing
// kernel); 1/2 is the factor of the two-for-one separation  C0 = (Z[f] + conj Z[D-f]) / 2,  C1 = (Z[f] - conj Z[D-f]) / 2i.
#pragma once

#include "rfsf_internal.h"

namespace rfsf {
namespace tuned {

// LDS index padding: one float2 of padding after every 16, so that the strided exchange of the
// Stockham passes and the contiguous accesses are both free of bank conflicts.
__host__ __device__ constexpr int pad(int e) { return e + (e >> 4); }

template <int LOG2D_, int LOG2R_ = 4>
struct Plan {
    static constexpr int LOG2D = LOG2D_;
    static constexpr int D = 1 << LOG2D;
    static constexpr int LOG2R = LOG2R_;
    static constexpr int kMinWaves = LOG2R_ > 4 ? 2 : 4;   // wavefronts per SIMD the register budget is set for
    static constexpr int R = 1 << LOG2R;        // points per lane
    static constexpr int G = D / R;             // lanes per transform
    static_assert(G <= 64, "a transform lives in one wavefront");
    static constexpr int FPW = 64 / G;          // transforms per wavefront
    static constexpr int GF = G;                // entries per fold round
    static constexpr int PD = D + D / 16;       // padded transform length in float2
    static constexpr int NP = LOG2D <= 4 ? 1 : (LOG2D <= 8 ? 2 : 3);
    static constexpr int radix(int p)
    {
        switch (LOG2D) {
            case 4: return 16;
            case 5: return p == 0 ? 16 : 2;
            case 6: return p == 0 ? 16 : 4;
            case 7: return p == 0 ? 16 : 8;
            case 8: return 16;
            case 9: return p == 1 ? 2 : 16;
            // three passes: the small radix goes in the middle, where all of a lane's butterflies
            // share their twiddles (Ns divides G), which keeps the twiddle registers few. D = 512 takes
            // 16 points per lane and a radix-2 middle pass rather than 32 points per lane and two passes:
            // half the registers and half the LDS per workgroup doubles the resident workgroups, which
            // outweighs the extra LDS exchange (measured: 20 % faster)
            case 10: return p == 1 ? 4 : 16;
            default: return p == 1 ? 8 : 16;    // 11 (32 points per lane)
        }
    }
    static constexpr int Ns(int p) { return p == 0 ? 1 : Ns(p - 1) * radix(p - 1); }
    // butterflies of pass p with distinct twiddles: butterfly u of a lane has k = (lg + G*u) mod Ns,
    // the same for every u when Ns divides G
    static constexpr int tw_sets(int p) { return G % Ns(p) == 0 ? 1 : R / radix(p); }
    // The twiddles of a radix-16 pass (15 per set) would cost 30 registers per set; they live in an
    // LDS table shared by the workgroup instead. Smaller passes keep theirs in registers.
    static constexpr bool tw_in_lds(int p) { return p > 0 && radix(p) >= 16; }
    static constexpr int tw_regs(int p) { return (p == 0 || tw_in_lds(p)) ? 0 : tw_sets(p) * (radix(p) - 1); }
    static constexpr int tw_lds(int p) { return tw_in_lds(p) ? tw_sets(p) * (radix(p) - 1) * G : 0; }   // float2 entries
    // array offsets of pass p: register twiddles (complex), LDS twiddles (float2) and write bases
    static constexpr int tw_off(int p) { return p <= 1 ? 0 : tw_off(p - 1) + tw_regs(p - 1); }
    static constexpr int twl_off(int p) { return p <= 1 ? 0 : twl_off(p - 1) + tw_lds(p - 1); }
    static constexpr int NTWL = twl_off(NP);
    static constexpr int wb_off(int p) { return p == 0 ? 0 : wb_off(p - 1) + R / radix(p - 1); }
    static constexpr int NTW = tw_off(NP) == 0 ? 1 : tw_off(NP);
    static constexpr int NWB = wb_off(NP);
    static constexpr int roff(int q) { return G >= 16 ? q * (G + G / 16) : tuned::pad(G * q); }
    static constexpr int pad(int e) { return tuned::pad(e); }     // position in a slot of element e
};

// Transform lengths 2^a 5^b that the paper's own experiments use as bucket counts (100, 200, 500, 1000): exact
// transforms of that length instead of a linear convolution in the next power of two above M (D - 1) + 1.
// 20 points per lane, D / 20 lanes per transform (the remaining lanes of a wavefront repeat the work of the
// first ones, see the kernel), passes of radix 10, 10 and 10 / 5 / 2 / none; slots are not padded; the
// twiddles of all passes after the first live in the LDS table. Selected as Plan<D>.
template <int DD>
struct MixedPlan {
    static constexpr int LOG2D = DD;
    static constexpr int D = DD;
    static constexpr int R = 20;
    static constexpr int G = D / R;
    static constexpr int FPW = 64 / G;
    static constexpr int GF = G;
    static constexpr int PD = D;
    static constexpr int NP = D == 100 ? 2 : 3;
    static constexpr int radix(int p) { return p < 2 ? 10 : (D == 1000 ? 10 : (D == 500 ? 5 : 2)); }
    static constexpr int Ns(int p) { return p == 0 ? 1 : Ns(p - 1) * radix(p - 1); }
    static constexpr int tw_sets(int p) { return G % Ns(p) == 0 ? 1 : R / radix(p); }
    static constexpr bool tw_in_lds(int p) { return p > 0; }
    static constexpr int tw_regs(int) { return 0; }
    static constexpr int tw_lds(int p) { return tw_in_lds(p) ? tw_sets(p) * (radix(p) - 1) * G : 0; }
    static constexpr int tw_off(int) { return 0; }
    static constexpr int twl_off(int p) { return p <= 1 ? 0 : twl_off(p - 1) + tw_lds(p - 1); }
    static constexpr int NTWL = twl_off(NP);
    static constexpr int wb_off(int p) { return p == 0 ? 0 : wb_off(p - 1) + R / radix(p - 1); }
    static constexpr int NTW = 1;
    static constexpr int NWB = wb_off(NP);
    static constexpr int roff(int q) { return G * q; }
    static constexpr int pad(int e) { return e; }
    static constexpr int kMinWaves = 4;
    static_assert(D % R == 0 && G * FPW <= 64, "");
};
template <> struct Plan<100> : MixedPlan<100> {};
template <> struct Plan<200> : MixedPlan<200> {};
template <> struct Plan<500> : MixedPlan<500> {};
template <> struct Plan<1000> : MixedPlan<1000> {};
// 2048 points in one wavefront: 32 points per lane (twice the registers, half the resident wavefronts, no barrier
// inside the transform). Selected as Plan<2048>.
template <> struct Plan<2048> : Plan<11, 5> {};

// Geometry of one LDS slot (float2 units): [0, ZS) data -- the staging area uses [0, 2F) and, because a
// direct load always deposits 128 coordinates, junk up to the next multiple of 128; the transform uses
// [0, PD) --, [ZS] a float2 that is always zero (source of buckets without a first or second coordinate).
__host__ __device__ constexpr int staged(int twoF) { return (twoF + 127) & ~127; }
__host__ __device__ constexpr int zero_slot(int PD, int twoF) { return PD > staged(twoF) ? PD : staged(twoF); }
__host__ __device__ constexpr int slot_stride(int PD, int twoF) { return (zero_slot(PD, twoF) + 2) & ~1; }

// Per-level table built once per call (uint32 words):
//   [0]                 NG, number of fold rounds
//   [64, 64 + D)        gather words: low 16 bits byte offset of the bucket's first coordinate in the
//                       staging area, high 16 bits of its second one (zero float2 if there is none)
//   [.., + 2F*G)        fold entries, G per round: low 16 bits byte offset of the coordinate to fold,
//                       high 16 bits byte offset of the first coordinate of its bucket (0xffff: padding)
struct TableLayout {
    int gather, fold, words;
};
__host__ __device__ inline TableLayout table_layout(int D, int G, int twoF)
{
    TableLayout t;
    t.gather = 64;
    t.fold = t.gather + D;
    t.words = (t.fold + twoF * G + 63) & ~63;
    return t;
}
constexpr uint32_t kFoldPad = 0xffffu;
constexpr int kFoldInRegs = 4;      // fold rounds whose entries are fetched with the other tables; later rounds load
                                    // theirs on the spot (4 measured best of 2, 4, 6, 8)

// cos(k pi / 16), k = 0..8
__device__ constexpr float kCos16[9] = {1.0f, 0.98078528040323043f, 0.92387953251128674f, 0.83146961230254524f,
                                        0.70710678118654752f, 0.55557023301960218f, 0.38268343236508977f,
                                        0.19509032201612825f, 0.0f};
constexpr float cos_pi16(int k) { return k <= 8 ? kCos16[k] : -kCos16[16 - k]; }   // k in [0, 16]
constexpr float sin_pi16(int k) { return k <= 8 ? kCos16[8 - k] : kCos16[k - 8]; }

constexpr int bitrev(int x, int bits)
{
    int r = 0;
    for (int i = 0; i < bits; ++i) r |= ((x >> i) & 1) << (bits - 1 - i);
    return r;
}
constexpr int ilog2(int n) { return n <= 1 ? 0 : 1 + ilog2(n / 2); }

// In-register forward DFT of N = 2..32 points, decimation in frequency; result k is left at
// position bitrev(k). Twiddles are compile-time constants; the trivial ones cost nothing.
template <int N, int BASE, int TOTAL>
__device__ __forceinline__ void dft_dif(float2 (&x)[TOTAL])
{
    if constexpr (N >= 2) {
        constexpr int H = N / 2;
#pragma unroll
        for (int i = 0; i < H; ++i) {
            const float2 a = x[BASE + i], b = x[BASE + i + H];
            x[BASE + i] = make_float2(a.x + b.x, a.y + b.y);
            const float dx = a.x - b.x, dy = a.y - b.y;
            const int k = i * (32 / N);                     // angle = k * pi / 16, k in [0, 16)
            if (k == 0) {
                x[BASE + i + H] = make_float2(dx, dy);
            } else if (k == 8) {                             // times -i
                x[BASE + i + H] = make_float2(dy, -dx);
            } else if (k == 4) {                             // times (1 - i) / sqrt 2
                x[BASE + i + H] = make_float2((dx + dy) * kCos16[4], (dy - dx) * kCos16[4]);
            } else if (k == 12) {                            // times (-1 - i) / sqrt 2
                x[BASE + i + H] = make_float2((dy - dx) * kCos16[4], -(dx + dy) * kCos16[4]);
            } else {                                         // times (c - i s)
                const float c = cos_pi16(k), s = sin_pi16(k);
                x[BASE + i + H] = make_float2(fmaf(dx, c, dy * s), fmaf(dy, c, -dx * s));
            }
        }
        dft_dif<H, BASE, TOTAL>(x);
        dft_dif<H, BASE + H, TOTAL>(x);
    }
}

__device__ __forceinline__ float2 cmulf(float2 a, float2 b)
{
    return make_float2(fmaf(a.x, b.x, -a.y * b.y), fmaf(a.x, b.y, a.y * b.x));
}
__device__ __forceinline__ float2 cfmaf(float2 a, float2 b, float2 c)   // a * b + c
{
    return make_float2(fmaf(a.x, b.x, fmaf(-a.y, b.y, c.x)), fmaf(a.x, b.y, fmaf(a.y, b.x, c.y)));
}

// In-register forward DFT of 5 points at x[B], x[B + ST], ..., natural order in and out.
template <int B, int ST, int TOTAL>
__device__ __forceinline__ void dft5(float2 (&x)[TOTAL])
{
    constexpr float c1 = 0.30901699437494742f, c2 = -0.80901699437494742f;    // cos(2 pi / 5), cos(4 pi / 5)
    constexpr float s1 = 0.95105651629515357f, s2 = 0.58778525229247313f;     // sin(2 pi / 5), sin(4 pi / 5)
    const float2 x0 = x[B], x1 = x[B + ST], x2 = x[B + 2 * ST], x3 = x[B + 3 * ST], x4 = x[B + 4 * ST];
    const float2 t1 = make_float2(x1.x + x4.x, x1.y + x4.y), t2 = make_float2(x2.x + x3.x, x2.y + x3.y);
    const float2 t3 = make_float2(x1.x - x4.x, x1.y - x4.y), t4 = make_float2(x2.x - x3.x, x2.y - x3.y);
    x[B] = make_float2(x0.x + t1.x + t2.x, x0.y + t1.y + t2.y);
    const float2 a1 = make_float2(fmaf(c1, t1.x, fmaf(c2, t2.x, x0.x)), fmaf(c1, t1.y, fmaf(c2, t2.y, x0.y)));
    const float2 a2 = make_float2(fmaf(c2, t1.x, fmaf(c1, t2.x, x0.x)), fmaf(c2, t1.y, fmaf(c1, t2.y, x0.y)));
    const float2 b1 = make_float2(fmaf(s1, t3.x, s2 * t4.x), fmaf(s1, t3.y, s2 * t4.y));
    const float2 b2 = make_float2(fmaf(s2, t3.x, -s1 * t4.x), fmaf(s2, t3.y, -s1 * t4.y));
    // X1 = a1 - i b1, X4 = a1 + i b1, X2 = a2 - i b2, X3 = a2 + i b2
    x[B + ST] = make_float2(a1.x + b1.y, a1.y - b1.x);
    x[B + 4 * ST] = make_float2(a1.x - b1.y, a1.y + b1.x);
    x[B + 2 * ST] = make_float2(a2.x + b2.y, a2.y - b2.x);
    x[B + 3 * ST] = make_float2(a2.x - b2.y, a2.y + b2.x);
}

// In-register forward DFT of 10 points, natural order in and out: one radix-2 stage (decimation in frequency),
// then the even outputs are the 5-point transform of the sums and the odd ones that of the twiddled differences.
__device__ __forceinline__ void dft10(float2 (&x)[10])
{
    constexpr float wc[5] = {1.0f, 0.80901699437494742f, 0.30901699437494742f, -0.30901699437494742f, -0.80901699437494742f};
    constexpr float ws[5] = {0.0f, 0.58778525229247313f, 0.95105651629515357f, 0.95105651629515357f, 0.58778525229247313f};
    float2 y[10];                                            // y[2 t] sums, y[2 t + 1] differences times exp(-2 pi i t / 10)
#pragma unroll
    for (int t = 0; t < 5; ++t) {
        const float2 a = x[t], b = x[t + 5];
        y[2 * t] = make_float2(a.x + b.x, a.y + b.y);
        const float dx = a.x - b.x, dy = a.y - b.y;
        y[2 * t + 1] = t == 0 ? make_float2(dx, dy) : make_float2(fmaf(dx, wc[t], dy * ws[t]), fmaf(dy, wc[t], -dx * ws[t]));
    }
    dft5<0, 2, 10>(y);                                       // y[2 k]     = X[2 k]
    dft5<1, 2, 10>(y);                                       // y[2 k + 1] = X[2 k + 1]
#pragma unroll
    for (int k = 0; k < 10; ++k) x[k] = y[k];
}

// Forward DFT of r points in registers; output k is left at position dft_out<r>(k).
template <int r>
__device__ __forceinline__ void dft_small(float2 (&x)[r])
{
    if constexpr (r == 10) dft10(x);
    else if constexpr (r == 5) dft5<0, 1, 5>(x);
    else dft_dif<r, 0, r>(x);
}
template <int r>
constexpr int dft_out(int k) { return (r & (r - 1)) == 0 ? bitrev(k, ilog2(r)) : k; }

// The same for a thread whose float2 are not complex numbers but two independent reals (pk; bins 0 and D/2
// of a real sequence's transform, which one thread carries in the two halves of its values): the products
// become componentwise. With pk false these are cmulf and cfmaf, operation for operation.
__device__ __forceinline__ float2 cmulf_pk(float2 a, float2 b, bool pk)
{
    const float s = pk ? 0.f : b.y, r = pk ? b.y : b.x;
    return make_float2(fmaf(a.x, b.x, -a.y * s), fmaf(a.x, s, a.y * r));
}
__device__ __forceinline__ float2 cfmaf_pk(float2 a, float2 b, float2 c, bool pk)
{
    const float s = pk ? 0.f : b.y, r = pk ? b.y : b.x;
    return make_float2(fmaf(a.x, b.x, fmaf(-a.y, s, c.x)), fmaf(a.x, s, fmaf(a.y, r, c.y)));
}

// Orders the LDS traffic of one wavefront: its LDS instructions execute in order, so only the
// compiler has to be kept from moving accesses across this point.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Exchange point inside a transform, which lives in one wavefront: a compiler-level ordering.
template <typename P>
__device__ __forceinline__ void transform_fence()
{
    wave_lds_fence();
}

// Per-lane constants of the wavefront-local FFT.
template <typename P>
struct WaveFft {
    float2 tw[P::NTW];
    int wbase[P::NWB];
    int rbase;
    const float2 *twl;      // LDS twiddle table of the radix-16 passes, entry ((set*(r-1) + t-1)*G + lg)

    __device__ __forceinline__ void init(int lg, float2 *twl_table)
    {
        rbase = P::pad(lg);
        twl = twl_table + lg;
        init_pass<0>(lg);
        fill_table<1>(twl_table);
    }

    // Workgroup-cooperative fill of the LDS twiddle table; the caller synchronises afterwards.
    template <int PI>
    __device__ __forceinline__ void fill_table(float2 *twl_table)
    {
        if constexpr (PI < P::NP) {
            if constexpr (P::tw_in_lds(PI)) {
                constexpr int r = P::radix(PI), Ns = P::Ns(PI);
                for (int i = threadIdx.x; i < P::tw_lds(PI); i += blockDim.x) {
                    const int l = i % P::G, ut = i / P::G, t = ut % (r - 1) + 1, u = ut / (r - 1);
                    const int k = (l + P::G * u) % Ns;
                    float s, c;
                    sincospif(-2.0f * (float)(k * t) / (float)(Ns * r), &s, &c);
                    twl_table[P::twl_off(PI) + i] = make_float2(c, s);
                }
            }
            fill_table<PI + 1>(twl_table);
        }
    }

    template <int PI>
    __device__ __forceinline__ void init_pass(int lg)
    {
        if constexpr (PI < P::NP) {
            constexpr int r = P::radix(PI), Ns = P::Ns(PI), NB = P::R / r;
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int j = lg + P::G * u;
                const int k = j % Ns;
                wbase[P::wb_off(PI) + u] = P::pad((j - k) * r + k);
            }
            if constexpr (PI > 0 && !P::tw_in_lds(PI)) {
                constexpr int NSETS = P::tw_sets(PI);
#pragma unroll
                for (int u = 0; u < NSETS; ++u) {
                    const int k = (lg + P::G * u) % Ns;
#pragma unroll
                    for (int t = 1; t < r; ++t) {
                        float s, c;
                        sincospif(-2.0f * (float)(k * t) / (float)(Ns * r), &s, &c);
                        tw[P::tw_off(PI) + u * (r - 1) + (t - 1)] = make_float2(c, s);
                    }
                }
            }
            init_pass<PI + 1>(lg);
        }
    }

    // Forward transform of the slot at `slot` (float2 LDS pointer, padded, natural order in and out).
    __device__ __forceinline__ void run(float2 *slot) const
    {
        float2 v[P::R];
#pragma unroll
        for (int q = 0; q < P::R; ++q) v[q] = slot[rbase + P::roff(q)];
        run_pass<0>(slot, v);
    }
    // The same with the input already in registers: v[q] is point lg + G*q of the lane's transform.
    __device__ __forceinline__ void run_from_registers(float2 *slot, float2 (&v)[P::R]) const
    {
        run_pass<0>(slot, v);
    }

    template <int PI>
    __device__ __forceinline__ void run_pass(float2 *slot, float2 (&v)[P::R]) const
    {
        if constexpr (PI < P::NP) {
            constexpr int r = P::radix(PI), Ns = P::Ns(PI), NB = P::R / r;
            transform_fence<P>();                    // every lane has its inputs in registers
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                float2 x[r];
#pragma unroll
                for (int t = 0; t < r; ++t) {
                    x[t] = v[u + t * NB];
                    if constexpr (PI > 0) {
                        constexpr int set = P::tw_sets(PI) == 1 ? 0 : 1;    // multiplier of u below
                        if (t > 0) {
                            if constexpr (P::tw_in_lds(PI)) {
                                x[t] = cmulf(x[t], twl[P::twl_off(PI) + ((set * u) * (r - 1) + (t - 1)) * P::G]);
                                if (t % 4 == 3) __builtin_amdgcn_sched_barrier(0);   // bound the twiddles in flight
                            } else {
                                x[t] = cmulf(x[t], tw[P::tw_off(PI) + (set * u) * (r - 1) + (t - 1)]);
                            }
                        }
                    }
                }
                dft_small<r>(x);
                float2 *dst = slot + wbase[P::wb_off(PI) + u];
#pragma unroll
                for (int t = 0; t < r; ++t) dst[P::pad(t * Ns)] = x[dft_out<r>(t)];
            }
            transform_fence<P>();
            if constexpr (PI + 1 < P::NP) {
#pragma unroll
                for (int q = 0; q < P::R; ++q) v[q] = slot[rbase + P::roff(q)];
                run_pass<PI + 1>(slot, v);
            }
        }
    }
};

// Number of transforms a workgroup has in flight per iteration (= its wavefronts when a transform lives in one
// wavefront). Normally one per level. With 5 or 6 levels that makes workgroups of 5 or 6 wavefronts, and the
// hardware then keeps far fewer of them resident than registers and LDS allow (measured with an empty kernel
// of the same footprint, ~116 registers and 51 KB: 1.7 workgroups = 8.6 wavefronts per CU for 5 wavefronts per
// workgroup, 15.6 wavefronts for 4 or 8 per workgroup: the dispatcher reserves registers for
// ceil(wavefronts / 4) wavefronts on every SIMD). For D = 1024 those level counts therefore run 8 wavefronts
// that take the (pair, level) transforms of the sequence in order, 8 at a time, whatever level they belong to.
// (Measured against one wavefront per level at 100 steps: D = 1024 +10 % with 5 levels, +23 % with 6, -9 to -15 %
// with 7; D = 512 +-1 %; D <= 256, where a wavefront carries four or more transforms, 35-60 % slower.) The
// same helps where one wavefront per level gives a CU too few wavefronts for other reasons: D = 1024 and 1000
// with up to three levels (+3-7 %; four levels: +-1 %), and D = 2048, whose slots let one workgroup per CU
// be resident whatever its size (up to seven levels: +10-20 %, one level +15 %, two +-0). D = 500 with 5 or 6
// levels gains 16 %, D = 512 with 5 levels 3 % (with 6: none); D = 256 loses 40 %.
__host__ __device__ constexpr int transforms_in_flight(int M, int LOG2D) {
    return ((LOG2D == 10 || LOG2D == 1000) && (M <= 3 || M == 5 || M == 6)) || (LOG2D == 2048 && M <= 7) ||
                   (LOG2D == 500 && (M == 5 || M == 6)) || (LOG2D == 9 && M == 5)
               ? 8 : M;
}

typedef const __attribute__((address_space(1))) uint32_t *GlobalWords;   // table words, known to be in global memory

constexpr size_t kLdsPerCu = 160 * 1024;
// LDS of a workgroup with NTR transforms in flight: their slots and the twiddle table of the plan.
__host__ __device__ constexpr size_t tuned_lds_bytes(int NTR, int FPW, int PD, int NTWL, int F)
{
    return sizeof(float2) * ((size_t)NTR * FPW * slot_stride(PD, 2 * F) + NTWL);
}

template <int LL>
struct LevelTag {
    static constexpr int value = LL;
};
// Calls f(LevelTag<l>) for a wavefront-uniform runtime level l in [0, M).
template <int M, int LL = 0, typename Fn>
__device__ __forceinline__ void with_level(int l, Fn &&f)
{
    if constexpr (LL + 1 < M) {
        if (l == LL) f(LevelTag<LL>{});
        else with_level<M, LL + 1>(l, f);
    } else {
        f(LevelTag<LL>{});
    }
}

// What level l of one pair hands to level l+1 of the same pair in the recurrence: the values of A_l before
// each of the two steps (p), with order >= 2 also those of A_{l-1} (q) and the transforms of level l (cp),
// with order 3 also those of A_{l-2} (r) and the transforms of level l-1 (cpp).
template <int ORDER>
struct LevelCarry {
    float2 p0, p1;
    float2 q0, q1, c0p, c1p;        // used with order >= 2
    float2 r0, r1, c0pp, c1pp;      // used with order 3
    __device__ __forceinline__ void reset()
    {
        p0 = p1 = make_float2(1.f, 0.f);
        q0 = q1 = c0p = c1p = r0 = r1 = c0pp = c1pp = make_float2(0.f, 0.f);
    }
};

// Items J = 0..NTR-1 of an iteration whose first item has level L0: calls f(LevelTag<level of item J>, LevelTag<J>,
// number of pair groups item J lies behind item 0).
template <int L0, int M, int NTR, int J = 0, typename Fn>
__device__ __forceinline__ void item_loop(Fn &&f)
{
    if constexpr (J < NTR) {
        f(LevelTag<(L0 + J) % M>{}, LevelTag<J>{}, (L0 + J) / M);
        item_loop<L0, M, NTR, J + 1>(f);
    }
}

// Calls f(LevelTag<0>), ..., f(LevelTag<M-1>).
template <int M, int LL = 0, typename Fn>
__device__ __forceinline__ void level_loop(Fn &&f)
{
    if constexpr (LL < M) {
        f(LevelTag<LL>{});
        level_loop<M, LL + 1>(f);
    }
}

// One level of one pair of time steps at one bin (Sec. 3.5 eq. (ts_rec)): z and zc are the transform of the
// level's slot at the bin and at its mirror image; separates the two real transforms and advances the bin's
// accumulator a = A_LL by both steps, c carrying what level LL - 1 of the same pair left. PK: the thread may be
// the packed one (pk), whose float2 hold bins 0 and D/2 and whose z, zc are Z[0], Z[D/2].
template <int ORDER, int LL, bool PK>
__device__ __forceinline__ void level_step(float2 z, float2 zc, bool pk, bool second_step, float2 &a, LevelCarry<ORDER> &c)
{
    auto mul = [&](float2 x, float2 y) { return PK ? cmulf_pk(x, y, pk) : cmulf(x, y); };
    auto fma = [&](float2 x, float2 y, float2 w) { return PK ? cfmaf_pk(x, y, w, pk) : cfmaf(x, y, w); };
    if constexpr (LL == 0) {
        c.reset();
        if (PK && pk) c.p0.y = c.p1.y = 1.f;                            // A_0 = 1 in both bins of the packed thread
    }
    // separation of the two real transforms; for the packed thread C = (2 Re z, 2 Re zc), (2 Im z, 2 Im zc):
    // the values the general formulas give at f = 0 and f = D/2
    float2 C0 = make_float2(z.x + zc.x, z.y - zc.y);
    // a second step that does not exist (odd number of increments) must contribute
    // exactly nothing; the separation alone would leave rounding noise of the first
    float2 C1 = make_float2(z.y + zc.y, zc.x - z.x);
    if constexpr (PK) {
        if (pk) {
            C0 = make_float2(z.x + z.x, zc.x + zc.x);
            C1 = make_float2(z.y + z.y, zc.y + zc.y);
        }
    }
    if (!second_step) C1 = make_float2(0.f, 0.f);
    const float2 a_old = a;
    float2 a_mid = fma(c.p0, C0, a_old);
    // order >= 2 (a time step may be used up to `order` times in a row, q equal indices weighted
    // 1/q!): also the values of levels l-2 (and l-3) before each step and the transforms of
    // levels l-1 (and l-2) at both steps
    float2 h0 = make_float2(0.f, 0.f), h1 = h0;
    if constexpr (ORDER >= 2 && LL > 0) {
        h0 = mul(c.c0p, C0);
        a_mid = fma(make_float2(0.5f * c.q0.x, 0.5f * c.q0.y), h0, a_mid);
    }
    if constexpr (ORDER >= 3 && LL > 1) {
        const float2 g = mul(c.c0pp, h0);
        a_mid = fma(make_float2(c.r0.x * (1.0f / 6.0f), c.r0.y * (1.0f / 6.0f)), g, a_mid);
    }
    float2 a_new = fma(c.p1, C1, a_mid);
    if constexpr (ORDER >= 2 && LL > 0) {
        h1 = mul(c.c1p, C1);
        a_new = fma(make_float2(0.5f * c.q1.x, 0.5f * c.q1.y), h1, a_new);
    }
    if constexpr (ORDER >= 3 && LL > 1) {
        const float2 g = mul(c.c1pp, h1);
        a_new = fma(make_float2(c.r1.x * (1.0f / 6.0f), c.r1.y * (1.0f / 6.0f)), g, a_new);
    }
    if constexpr (ORDER >= 3) {
        c.r0 = c.q0;
        c.r1 = c.q1;
        c.c0pp = c.c0p;
        c.c1pp = c.c1p;
    }
    if constexpr (ORDER >= 2) {
        c.q0 = c.p0;
        c.q1 = c.p1;
        c.c0p = C0;
        c.c1p = C1;
    }
    a = a_new;
    c.p0 = a_old;
    c.p1 = a_mid;
}

// Wavefronts per SIMD the register budget of the kernel is set for: the plan's, except that workgroups of 5 or 6
// wavefronts with 6 to 12 transforms per wavefront (D = 100, 128, 200) get 96 registers: their workgroups then
// find room on a CU more often (see transforms_in_flight; measured +8-15 %).
template <int LOG2D, int M>
constexpr int kernel_min_waves()
{
    using P = Plan<LOG2D>;
    return (P::FPW > 4 && P::FPW < 16 && (M == 5 || M == 6)) ? 5 : P::kMinWaves;
}

template <int LOG2D, int M, int ORDER, int NTR>
__global__ __launch_bounds__(64 * NTR)
    __attribute__((amdgpu_waves_per_eu(kernel_min_waves<LOG2D, M>(), kernel_min_waves<LOG2D, M>() > 4 ? 8 : 4))) void sketch_fft_scan_kernel(
    const float *__restrict__ dphi, const uint32_t *__restrict__ table, int64_t L,
    const int64_t *__restrict__ lengths, int F, int Dout, float *__restrict__ out, int64_t ld_out, TimeCut cut)
{
    using P = Plan<LOG2D>;
    // kStream: the workgroup's NTR transforms of an iteration are the next NTR (pair group, level) items of the
    // sequence in that order, so a wavefront changes level from iteration to iteration and an iteration
    // may end in the middle of a pair; otherwise transform w of the workgroup is always level w.
    constexpr bool kStream = NTR != M;
    static_assert(!kStream || NTR > M, "streaming needs a slot per level");
    // Bins of phase 3: f = 0 .. D/2, thread t owning f = t, t + NT, ... The transforms of real sequences are real
    // at f = 0 and f = D/2. Where that saves a bin per thread (NT divides D/2), thread 0 carries both in one
    // float2 (bin 0 in .x, bin D/2 in .y; kPack) and the bins are f = 0 .. D/2 - 1.
    constexpr int D = P::D, NT = 64 * NTR;
    constexpr bool kPack = (D / 2) % NT == 0;
    constexpr int NB = kPack ? D / 2 : D / 2 + 1, BPT = (NB + NT - 1) / NT;
    // Phase 3 is compiled separately for iterations in which every item exists and has both time steps (no
    // per-item conditions and selects) when a wavefront has at most two transforms per iteration; with more the
    // extra copy costs registers.
    constexpr bool kSplitFull = P::FPW <= 2;
    extern __shared__ float2 lds[];                    // [NTR][FPW][PS] slots, then the twiddle table
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wv = wave;                                     // transform of the workgroup
    // lanes beyond the G * FPW that the wavefront's transforms occupy (lengths that are no power of two) repeat the
    // work of the first ones: same addresses, same values
    constexpr int kLanesUsed = P::G * P::FPW;
    const int lane_t = kLanesUsed < 64 && lane >= kLanesUsed ? lane - kLanesUsed : lane;
    const int slot_id = lane_t / P::G;
    const int lg = lane_t % P::G;                            // lane within the transform
    const int twoF = 2 * F;
    const int ZS = zero_slot(P::PD, twoF), PS = slot_stride(P::PD, twoF);
    float2 *twl_table = lds + (size_t)NTR * P::FPW * PS;        // behind the slots
    float2 *wave_lds = lds + (size_t)wv * P::FPW * PS;
    float2 *my_slot = wave_lds + slot_id * PS;
    char *my_slot_bytes = reinterpret_cast<char *>(my_slot);
    // the workgroup's row of out, its sequence and its piece of that sequence (one piece: the whole sequence)
    const int64_t row_id = blockIdx.x;
    const int64_t n = cut.pieces == 1 ? row_id : row_id / cut.pieces, piece = row_id - n * cut.pieces;
    // this sequence's own number of points (variable-length batch: X is padded to L points, the steps beyond a
    // sequence's length do not exist); out-of-range entries are clamped, they are never used as addresses
    const int64_t Ln = lengths ? (lengths[n] < 1 ? 1 : (lengths[n] > L ? L : lengths[n])) : L;
    // the piece's own steps: 2 * cut.pairs of them from its first one on, fewer (or none) at the sequence's end
    const int64_t steps_left = Ln - 1 - 2 * piece * cut.pairs;
    const int64_t T = cut.mode == 2 || steps_left < 0 ? 0 : (steps_left < 2 * cut.pairs ? steps_left : 2 * cut.pairs);
    const int64_t pairs = (T + 1) / 2;
    // pair p of level l: 2F float2 at seq + l * 2 * twoF + p * pf (pair layout of the producing kernel, Lp / 2
    // pair slots per sequence with Lp = L rounded up to even)
    const int64_t pf = (int64_t)cut.row_levels * 2 * twoF;
    const float *seq = dphi + (n * ((L + 1) / 2) + piece * cut.pairs) * pf;
    const TableLayout tl = table_layout(D, P::GF, twoF);
    const int nload = staged(twoF) / 128;                    // direct loads per pair, 128 coordinates each
    // one level per wavefront for good: its increments, table and number of fold rounds
    const float *seq_fixed = seq + (int64_t)wv * 2 * twoF;
    const uint32_t *tab_fixed = table + (int64_t)wv * tl.words;
    const int NG_fixed = kStream ? 0 : (int)tab_fixed[0];

    WaveFft<P> fft;
    fft.init(lg, twl_table);
    if (lg == 0) my_slot[ZS] = make_float2(0.f, 0.f);
    __syncthreads();

    float2 A[BPT][M];
#pragma unroll
    for (int b = 0; b < BPT; ++b)
#pragma unroll
        for (int l = 0; l < M; ++l) A[b][l] = make_float2(0.f, 0.f);
    // accumulators kept outside the kernel (sequences cut in time): M levels of bins 0 .. D/2 per row
    float2 *spectra_row = cut.mode != 0 ? cut.spectra + row_id * (int64_t)(M * (D / 2 + 1)) : nullptr;
    if (cut.mode == 2) {
#pragma unroll
        for (int b = 0; b < BPT; ++b) {
            const int f = tid + NT * b;
            if (f < NB) {
#pragma unroll
                for (int l = 0; l < M; ++l) {
                    const float2 *sp = spectra_row + l * (D / 2 + 1);
                    A[b][l] = kPack && f == 0 ? make_float2(sp[0].x, sp[D / 2].x) : sp[f];
                }
            }
        }
    }

    // Staging: pair pair0 + s of level lvl goes to slot s of the wavefront, 128 coordinates (1 KB) per
    // instruction, lane i supplying coordinates 2i and 2i+1. Pairs beyond the last one (final group only) are redirected to the last pair and
    // ignored later; coordinates beyond 2F read the following floats of the workspace (which is padded at its
    // end for this) and land in the unused part of the staging area.
    auto stage_direct = [&](int lvl, int64_t pair0) {
#pragma unroll
        for (int s = 0; s < P::FPW; ++s) {
            const int64_t p = pair0 + s < pairs ? pair0 + s : pairs - 1;
            const float *src = (kStream ? seq + (int64_t)lvl * 2 * twoF : seq_fixed) + p * pf + 4 * lane;
            float2 *dst = wave_lds + s * PS;
            for (int j = 0; j < nload; ++j)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + 256 * j),
                                                 (__attribute__((address_space(3))) void *)(dst + 128 * j), 16, 0, 0);
        }
    };

    // Early staging: when the transforms of one iteration fit a thread's registers (ZREGS float2), phase 3 first
    // copies them out of LDS, the slots are released by the second barrier at once, and the next iteration's
    // direct loads are issued before the recurrence arithmetic, which then runs under their latency.
    // (Measured: 3-4 % on D = 1024 and 2048 with five levels; with 32 float2 -- D = 512, four levels -- it no
    // longer pays, and loading the next iteration's table words early as well costs more registers than it hides.)
    constexpr int ZREGS = P::FPW * BPT * NTR * 2;
    constexpr bool kEarly = ZREGS <= (P::kMinWaves <= 2 ? 64 : 24);    // (a plan with twice the registers per wavefront affords more)
    uint32_t gw[P::R], fw[kFoldInRegs];

    // The item of this wavefront: level and first pair of its transform in the current iteration (a transform
    // carries FPW consecutive pairs of one level, a pair group). Streaming: the items of the sequence are counted
    // (group, level) with the level running fastest, and this wavefront has number iteration * NTR + wv.
    int lvl = kStream ? wv % M : wv;
    int64_t pair0 = kStream ? (wv / M) * P::FPW : 0;
    auto advance = [&](int &l, int64_t &p0) {                // the same wavefront's item one iteration later
        if constexpr (kStream) {
            l += NTR % M;
            p0 += (NTR / M) * P::FPW;
            if (l >= M) {
                l -= M;
                p0 += P::FPW;
            }
        } else {
            p0 += P::FPW;
        }
    };
    // first item of the iteration (the one of wavefront 0; streaming only)
    int lvl_first = 0;
    int64_t pair0_first = 0;
    LevelCarry<ORDER> carry[kStream ? P::FPW : 1][kStream ? BPT : 1];

    __builtin_amdgcn_s_setprio(1);
    if (kEarly && pair0 < pairs) stage_direct(lvl, pair0);
    // an iteration exists while its first item does
    while ((kStream ? pair0_first : pair0) < pairs) {
        if (!kStream || pair0 < pairs) {                      // streaming: the last iteration may have fewer items
            // Tables of this level. They are the same whenever the level comes up and stay in L1/L2; the
            // pointer is laundered so that the compiler reloads them every iteration instead of keeping ~90
            // loop-invariant registers (table words and everything derived from them) alive across the transform.
            const uint32_t *tabl = kStream ? table + (int64_t)lvl * tl.words : tab_fixed;
            asm volatile("" : "+s"(tabl));
            // (the laundered pointer would be a generic one: loads through it would count as LDS operations too)
            const GlobalWords tabi = (GlobalWords)tabl;
            const int NG = kStream ? (int)tabi[0] : NG_fixed;
#pragma unroll
            for (int q = 0; q < P::R; ++q) gw[q] = tabi[tl.gather + lg + P::G * q];
#pragma unroll
            for (int g = 0; g < kFoldInRegs; ++g) fw[g] = g < NG ? tabi[tl.fold + g * P::GF + (lg % P::GF)] : kFoldPad << 16;

            // 1a. staging
            if (!kEarly) stage_direct(lvl, pair0);
            __builtin_amdgcn_s_waitcnt(0x0f70);                 // vmcnt(0): the direct loads have landed
            if ((T & 1) && pair0 + P::FPW >= pairs) {
                // odd number of increments, last pair: its second step does not exist; what the producer left in
                // its place (the increment across the sequence boundary) is cleared so that it cannot touch the result
                float2 *st = wave_lds + (int)(pairs - 1 - pair0) * PS;
                for (int a = lane; a < twoF; a += 64) st[a].y = 0.f;
            }
            transform_fence<P>();
            // 1b. fold the third and later coordinates of a bucket into its first one, one rank per round
            auto fold = [&](uint32_t w) {
                const uint32_t own = w & 0xffffu, tgt = w >> 16;
                if (tgt != kFoldPad) {
                    const float2 x = *reinterpret_cast<const float2 *>(my_slot_bytes + own);
                    const float2 y = *reinterpret_cast<const float2 *>(my_slot_bytes + tgt);
                    *reinterpret_cast<float2 *>(my_slot_bytes + tgt) = make_float2(x.x + y.x, x.y + y.y);
                }
                wave_lds_fence();
            };
#pragma unroll
            for (int g = 0; g < kFoldInRegs; ++g)
                if (g < NG) fold(fw[g]);
            for (int g = kFoldInRegs; g < NG; ++g) fold(tabi[tl.fold + g * P::GF + (lg % P::GF)]);
            // 1c. gather: first and second coordinate of each of this lane's buckets
            float2 v[P::R];
#pragma unroll
            for (int q = 0; q < P::R; ++q) {
                const float2 x0 = *reinterpret_cast<const float2 *>(my_slot_bytes + (gw[q] & 0xffffu));
                const float2 x1 = *reinterpret_cast<const float2 *>(my_slot_bytes + (gw[q] >> 16));
                v[q] = make_float2(x0.x + x1.x, x0.y + x1.y);
                // keep the scheduler from issuing all 2R reads at once (it would need 4R registers)
                if (q % 4 == 3) __builtin_amdgcn_sched_barrier(0);
            }
            // 2. FPW transforms per wavefront, in place in the slots. The transform is the one long stretch of
            // arithmetic of an iteration; everything else is short pieces of work between waits (loads, LDS round
            // trips, barriers). A wavefront in those phases runs at a raised priority, so that it gets its few
            // instructions issued at once and goes back to waiting instead of queueing behind other wavefronts'
            // transforms (measured: 3-7 % on every workload; the other way round, 2-3 % slower).
            __builtin_amdgcn_s_setprio(0);
            fft.run_from_registers(my_slot, v);
            __builtin_amdgcn_s_setprio(1);
        }
        __syncthreads();
        // 3. per-bin separation and recurrence, two time steps per slot, items in order (levels ascending
        // within a pair).
        // For D = 1024 (128-register budget, one pair per wavefront) the thread index is laundered so that
        // the LDS addresses of the bins are recomputed here (a few adds) instead of being kept across the
        // whole iteration as loop invariants, where they were spilled to scratch (measured: 8 % faster
        // there, slower for the other transform lengths).
        int tid_here = tid;
        if constexpr (LOG2D == 10 || LOG2D == 1000) asm volatile("" : "+v"(tid_here));
        float2 zreg[kEarly ? P::FPW : 1][kEarly ? BPT : 1][kEarly ? NTR : 1][2];
        if constexpr (kEarly) {
#pragma unroll
            for (int s = 0; s < P::FPW; ++s)
#pragma unroll
                for (int b = 0; b < BPT; ++b) {
                    const int f = tid_here + NT * b;
                    const int fi = P::pad(f < NB ? f : 0);
                    const int fc = kPack ? P::pad(f > 0 && f < NB ? D - f : D / 2) : P::pad(f > 0 && f < NB ? D - f : 0);
#pragma unroll
                    for (int j = 0; j < NTR; ++j) {
                        const float2 *Z = lds + ((size_t)j * P::FPW + s) * PS;
                        zreg[s][b][j][0] = Z[fi];
                        zreg[s][b][j][1] = Z[fc];
                    }
                }
            __syncthreads();                                        // the slots are free again
        }
        const int64_t pair0_now = pair0;
        advance(lvl, pair0);
        if (kEarly && pair0 < pairs) stage_direct(lvl, pair0);

        // one (pair, level) of one bin: separation of the two steps and A_LL += ... for both
        auto update_bin = [&](auto level_tag, auto packed_tag, auto full_tag, int s, int b, int j, int64_t pair0_j,
                              LevelCarry<ORDER> &c) {
            constexpr int LL = decltype(level_tag)::value;
            constexpr bool PK = kPack && decltype(packed_tag)::value != 0;   // this wavefront holds the thread of bins 0 and D/2
            constexpr bool FULL = decltype(full_tag)::value != 0;      // every item of the iteration has both steps
            const int f = tid_here + NT * b;                            // a bin that exists (the caller checks)
            const bool pk = PK && b == 0 && f == 0;
            const bool second_step = FULL || 2 * (pair0_j + s) + 1 < T;    // wavefront-uniform
            float2 z, zc;
            if constexpr (kEarly) {
                z = zreg[s][b][j][0];
                zc = zreg[s][b][j][1];
            } else {
                const float2 *Z = lds + ((size_t)j * P::FPW + s) * PS;
                z = Z[P::pad(f)];
                zc = Z[kPack ? P::pad(f > 0 ? D - f : D / 2) : P::pad(f > 0 ? D - f : 0)];
            }
            level_step<ORDER, LL, PK>(z, zc, pk, second_step, A[b][LL], c);
        };
        // The whole of phase 3, compiled four times: for the wavefront of the packed thread and for the others,
        // and for iterations whose items all exist and have both time steps (all but the last one or two of a
        // sequence: no per-item conditions, no selects) and for the rest.
        auto phase3 = [&](auto packed_tag, auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value != 0;
            if constexpr (kStream) {
                // one branch on the level of the iteration's first item; inside it every item's level is static
                with_level<M>(lvl_first, [&](auto first_tag) {
                    constexpr int L0 = decltype(first_tag)::value;
                    item_loop<L0, M, NTR>([&](auto level_tag, auto item_tag, int group_offset) {
                        constexpr int j = decltype(item_tag)::value;
                        const int64_t pair0_j = pair0_first + group_offset * P::FPW;
                        if (FULL || pair0_j < pairs) {
#pragma unroll
                            for (int s = 0; s < P::FPW; ++s) {
                                if (!FULL && pair0_j + s >= pairs) continue;   // slot without a pair (last group only)
#pragma unroll
                                for (int b = 0; b < BPT; ++b)
                                    if (NT * BPT == NB || tid_here + NT * b < NB)
                                        update_bin(level_tag, packed_tag, full_tag, s, b, j, pair0_j, carry[s][b]);
                            }
                        }
                    });
                });
            } else {
                // with more than four transforms per wavefront and three or more levels the loop over the pairs
                // stays a loop: unrolled it needs 50-150 spilled registers (measured rolled: D = 64 ... 200 with
                // 4-8 levels 1.4-3 times faster; with one or two levels up to 45 % slower, hence the condition)
#pragma unroll(P::FPW > 4 && M >= 3 ? 1 : P::FPW)
                for (int s = 0; s < P::FPW; ++s) {
                    if (!FULL && pair0_now + s >= pairs) continue;             // slot without a pair (last iteration only)
#pragma unroll
                    for (int b = 0; b < BPT; ++b) {
                        if (NT * BPT == NB || tid_here + NT * b < NB) {
                            LevelCarry<ORDER> c;
                            level_loop<M>([&](auto level_tag) {
                                update_bin(level_tag, packed_tag, full_tag, s, b, decltype(level_tag)::value, pair0_now, c);
                            });
                        }
                    }
                }
            }
        };
        // full: the last pair of the last pair group that this iteration touches has a second step
        const int64_t last_pair0 = kStream ? pair0_first + ((lvl_first + NTR - 1) / M) * P::FPW : pair0_now;
        const bool full = 2 * (last_pair0 + P::FPW) - 1 < T;
        if (kPack && wave == 0) {
            if (kSplitFull && full) phase3(LevelTag<1>{}, LevelTag<1>{});
            else phase3(LevelTag<1>{}, LevelTag<0>{});
        } else {
            if (kSplitFull && full) phase3(LevelTag<0>{}, LevelTag<1>{});
            else phase3(LevelTag<0>{}, LevelTag<0>{});
        }
        if constexpr (kStream) advance(lvl_first, pair0_first);
        if (!kEarly) __syncthreads();
    }
    if (kEarly) __syncthreads();

    if (cut.mode == 1) {                                     // a piece of a sequence: its accumulators are the result
#pragma unroll
        for (int b = 0; b < BPT; ++b) {
            const int f = tid + NT * b;
            if (f < NB) {
#pragma unroll
                for (int l = 0; l < M; ++l) {
                    float2 *sp = spectra_row + l * (D / 2 + 1);
                    const float2 y = A[b][l];
                    if (kPack && f == 0) {                   // bins 0 and D/2, both real
                        sp[0] = make_float2(y.x, 0.f);
                        sp[D / 2] = make_float2(y.y, 0.f);
                    } else {
                        sp[f] = y;
                    }
                }
            }
        }
        return;
    }

    // Phi_m = Re(FFT(conj Y_m)) / D with Y_m the Hermitian extension of A_m; slot 0 of transform m of the workgroup.
#pragma unroll
    for (int b = 0; b < BPT; ++b) {
        const int f = tid + NT * b;
        if (f < NB) {
#pragma unroll
            for (int l = 0; l < M; ++l) {
                float2 *Y = lds + (size_t)l * P::FPW * PS;
                const float2 y = A[b][l];
                if (kPack && f == 0) {                       // bins 0 and D/2, both real
                    Y[P::pad(0)] = make_float2(y.x, 0.f);
                    Y[P::pad(D / 2)] = make_float2(y.y, 0.f);
                } else {
                    Y[P::pad(f)] = make_float2(y.x, -y.y);
                    if (f > 0 && f < D / 2) Y[P::pad(D - f)] = y;
                }
            }
        }
    }
    __syncthreads();
    if (wv < M) {                                            // (always, unless streaming)
        fft.run(my_slot);
        transform_fence<P>();
        float *row = out + row_id * ld_out;
        if (tid == 0) row[0] = 1.0f;
        const float invD = 1.0f / (float)D;
        // Dout buckets per level. Dout == D: the transform was circular in D already. Dout < D (a bucket
        // count that is no power of two): D was chosen so large that the M-fold convolution never wrapped,
        // and the linear result is folded modulo Dout here.
        for (int j = lane; j < Dout; j += 64) {
            float acc = 0.f;
            for (int e = j; e < D; e += Dout) acc += wave_lds[P::pad(e)].x;
            row[1 + (int64_t)wv * Dout + j] = acc * invD;
        }
    }
}

}  // namespace tuned
}  // namespace rfsf
