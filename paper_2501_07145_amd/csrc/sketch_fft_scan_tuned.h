// Tuned kernel for steps 3-4 (CountSketch, Fourier-domain level recursion over time, inverse
// transform; Sec. 3.5, eqs. (cs), (ts_def), (ts_rec) with p = 1).
//
// Work decomposition (one workgroup per sequence, M wavefronts, wavefront m owns level m):
//   per iteration every wavefront handles FPW pairs of consecutive time steps of its level:
//     1. clears its LDS slots and scatter-adds the signed increments of the 2*FPW time steps
//        into them (step 2k goes to the real parts, step 2k+1 to the imaginary parts of slot
//        k). LDS float atomics cost about three cycles per lane on this chip, so conflicts are
//        handled wavefront-locally instead: the 2F coordinates are taken 64 at a time; a
//        precomputed level says how many earlier coordinates of the same 64 share the bucket.
//        Level-0 lanes hit distinct buckets and do a plain read-add-write; for D <= 512 the
//        level-1 lanes do the same in a second masked round; the rare rest uses ds_add_f32.
//        Successive groups of 64 are ordered by the in-order LDS queue of the wavefront,
//     2. runs FPW complex FFTs of length D held in its own LDS slots, G = D/R lanes per
//        transform with R points per lane in registers (Stockham passes, radix up to 32 in
//        registers, one LDS exchange per pass, no workgroup barrier inside the transform),
//   then, after one barrier, every thread owns a few frequency bins, separates the two real
//   transforms of each slot, and advances the accumulators A_1..A_M of its bins by the two
//   time steps (A_m += A_{m-1}(before the step) * C_m, A_0 = 1).
//   After the last time step, wavefront m transforms A_m back and writes block m of the row.
//
// The increments arrive pre-multiplied by 1/2 (done by the producing kernel), which is the
// factor of the two-for-one separation  C0 = (Z[f] + conj Z[D-f]) / 2,  C1 = (Z[f] - conj Z[D-f]) / 2i.
#pragma once

#include "rfsf_internal.h"

namespace rfsf {
namespace tuned {

// LDS index padding: one float2 of padding after every 16, so that the strided exchange of the
// Stockham passes and the contiguous accesses are both free of bank conflicts.
__host__ __device__ constexpr int pad(int e) { return e + (e >> 4); }

template <int LOG2D_>
struct Plan {
    static constexpr int LOG2D = LOG2D_;
    static constexpr int D = 1 << LOG2D;
    static constexpr int LOG2R = (LOG2D == 9 || LOG2D == 11) ? 5 : 4;
    static constexpr int R = 1 << LOG2R;        // points per lane
    static constexpr int G = D / R;             // lanes per transform
    static constexpr int FPW = 64 / G;          // transforms per wavefront
    static constexpr int PD = D + D / 16;       // padded transform length in float2
    static constexpr int PS = PD + 64;          // slot stride: one spare float2 per lane behind the data
    static constexpr int LOADB = FPW >= 8 ? 1 : 8 / FPW;   // 64-coordinate groups loaded per batch
    static constexpr int NP = LOG2D <= 4 ? 1 : (LOG2D <= 9 ? 2 : 3);
    static constexpr int radix(int p)
    {
        switch (LOG2D) {
            case 4: return 16;
            case 5: return p == 0 ? 16 : 2;
            case 6: return p == 0 ? 16 : 4;
            case 7: return p == 0 ? 16 : 8;
            case 8: return 16;
            case 9: return p == 0 ? 32 : 16;
            // three passes: the small radix goes in the middle, where all of a lane's butterflies
            // share their twiddles (Ns divides G), which keeps the twiddle registers few
            case 10: return p == 1 ? 4 : 16;
            default: return p == 1 ? 8 : 16;    // 11
        }
    }
    static constexpr int Ns(int p) { return p == 0 ? 1 : Ns(p - 1) * radix(p - 1); }
    // butterflies of pass p with distinct twiddles: butterfly u of a lane has k = (lg + G*u) mod Ns,
    // the same for every u when Ns divides G
    static constexpr int tw_sets(int p) { return G % Ns(p) == 0 ? 1 : R / radix(p); }
    // register-array offsets of pass p: twiddles (complex) and write bases
    static constexpr int tw_off(int p) { return p <= 1 ? 0 : tw_off(p - 1) + tw_sets(p - 1) * (radix(p - 1) - 1); }
    static constexpr int wb_off(int p) { return p == 0 ? 0 : wb_off(p - 1) + R / radix(p - 1); }
    static constexpr int NTW = NP == 1 ? 1 : tw_off(NP);
    static constexpr int NWB = wb_off(NP);
    static constexpr int roff(int q) { return G >= 16 ? q * (G + G / 16) : pad(G * q); }
};

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

// Orders the LDS traffic of one wavefront: its LDS instructions execute in order, so only the
// compiler has to be kept from moving accesses across this point.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Per-lane constants of the wavefront-local FFT.
template <typename P>
struct WaveFft {
    float2 tw[P::NTW];
    int wbase[P::NWB];
    int rbase;

    __device__ __forceinline__ void init(int lg)
    {
        rbase = pad(lg);
        init_pass<0>(lg);
    }

    template <int PI>
    __device__ __forceinline__ void init_pass(int lg)
    {
        if constexpr (PI < P::NP) {
            constexpr int r = P::radix(PI), Ns = P::Ns(PI), NB = P::R / r;
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int j = lg + P::G * u;
                const int k = j & (Ns - 1);
                wbase[P::wb_off(PI) + u] = pad((j - k) * r + k);
            }
            if constexpr (PI > 0) {
                constexpr int NSETS = P::tw_sets(PI);
#pragma unroll
                for (int u = 0; u < NSETS; ++u) {
                    const int k = (lg + P::G * u) & (Ns - 1);
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

    template <int PI>
    __device__ __forceinline__ void run_pass(float2 *slot, float2 (&v)[P::R]) const
    {
        if constexpr (PI < P::NP) {
            constexpr int r = P::radix(PI), Ns = P::Ns(PI), NB = P::R / r, LR = ilog2(r);
            wave_lds_fence();                    // every lane has its inputs in registers
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                float2 x[r];
#pragma unroll
                for (int t = 0; t < r; ++t) {
                    x[t] = v[u + t * NB];
                    if constexpr (PI > 0) {
                        if (t > 0) x[t] = cmulf(x[t], tw[P::tw_off(PI) + (P::tw_sets(PI) == 1 ? 0 : u) * (r - 1) + (t - 1)]);
                    }
                }
                dft_dif<r, 0, r>(x);
                float2 *dst = slot + wbase[P::wb_off(PI) + u];
#pragma unroll
                for (int t = 0; t < r; ++t) dst[pad(t * Ns)] = x[bitrev(t, LR)];
            }
            wave_lds_fence();
            if constexpr (PI + 1 < P::NP) {
#pragma unroll
                for (int q = 0; q < P::R; ++q) v[q] = slot[rbase + P::roff(q)];
                run_pass<PI + 1>(slot, v);
            }
        }
    }
};

// Packed table entry: bits 0-15 float2 index of the bucket inside a padded slot, bits 16-17
// collision level inside the group of 64 coordinates (0, 1, 2 = two or more earlier ones,
// 3 = no coordinate), bit 31 the sign.
constexpr uint32_t kSkipEntry = 3u << 16;

template <int LOG2D, int M>
__global__ __launch_bounds__(64 * M) __attribute__((amdgpu_waves_per_eu(Plan<LOG2D>::LOG2R == 4 ? 4 : 2, 4))) void sketch_fft_scan_kernel(
    const float *__restrict__ dphi, const uint32_t *__restrict__ table, int64_t L, int F,
    float *__restrict__ out, int64_t ld_out)
{
    using P = Plan<LOG2D>;
    constexpr int D = P::D, NT = 64 * M, NB = D / 2 + 1, BPT = (NB + NT - 1) / NT;
    extern __shared__ float2 lds[];                    // [M][FPW][PS]
    const int tid = threadIdx.x, lane = tid & 63, m = tid >> 6;
    const int slot_id = lane / P::G, lg = lane % P::G;
    float2 *wave_lds = lds + (size_t)m * P::FPW * P::PS;
    float2 *my_slot = wave_lds + slot_id * P::PS;
    const int64_t n = blockIdx.x, T = L - 1;
    const int twoF = 2 * F;
    const int64_t rf = (int64_t)M * twoF;
    const float *seq = dphi + n * L * rf + (int64_t)m * twoF;   // row k of this level: seq + k * rf
    const uint32_t *tab = table + (int64_t)m * twoF;

    WaveFft<P> fft;
    fft.init(lg);

    float2 A[BPT][M];
#pragma unroll
    for (int b = 0; b < BPT; ++b)
#pragma unroll
        for (int l = 0; l < M; ++l) A[b][l] = make_float2(0.f, 0.f);

    const int64_t pairs = (T + 1) / 2;
    for (int64_t pair0 = 0; pair0 < pairs; pair0 += P::FPW) {
        // 1. clear this wavefront's slots, then signed scatter-add of 2*FPW time steps
        for (int i = lane; i < P::FPW * P::PS; i += 64) wave_lds[i] = make_float2(0.f, 0.f);
        wave_lds_fence();
        for (int a0 = 0; a0 < twoF; a0 += 64 * P::LOADB) {
            uint32_t tb[P::LOADB];
            float2 val[P::LOADB][P::FPW];
            // all global loads of the batch are issued before the first use
#pragma unroll
            for (int b = 0; b < P::LOADB; ++b) {
                const int a = a0 + 64 * b + lane;
                const bool ok = a < twoF;
                const int aa = ok ? a : twoF - 1;
                const uint32_t t = tab[aa];
                tb[b] = ok ? t : kSkipEntry;
                const uint32_t sgn = t & 0x80000000u;
#pragma unroll
                for (int s = 0; s < P::FPW; ++s) {
                    const int64_t k0 = 2 * (pair0 + s);
                    const int64_t kk0 = k0 < T ? k0 : T - 1, kk1 = k0 + 1 < T ? k0 + 1 : T - 1;
                    const float x0 = __uint_as_float(__float_as_uint(seq[kk0 * rf + aa]) ^ sgn);
                    const float x1 = __uint_as_float(__float_as_uint(seq[kk1 * rf + aa]) ^ sgn);
                    val[b][s] = make_float2(k0 < T ? x0 : 0.f, k0 + 1 < T ? x1 : 0.f);
                }
            }
#pragma unroll
            for (int b = 0; b < P::LOADB; ++b) {
                const uint32_t lvl = (tb[b] >> 16) & 3u;
                const int off = (int)(tb[b] & 0xffffu);
                // round 0: every lane issues; lanes of other levels use their spare float2
                const int sel = lvl == 0 ? off : P::PD + lane;
                float2 old[P::FPW];
#pragma unroll
                for (int s = 0; s < P::FPW; ++s) old[s] = wave_lds[s * P::PS + sel];
#pragma unroll
                for (int s = 0; s < P::FPW; ++s)
                    wave_lds[s * P::PS + sel] = make_float2(old[s].x + val[b][s].x, old[s].y + val[b][s].y);
                wave_lds_fence();
                if constexpr (P::LOG2D <= 9) {        // collisions inside a group of 64 are common
                    if (lvl == 1) {                   // second coordinate of a bucket inside this group
#pragma unroll
                        for (int s = 0; s < P::FPW; ++s) old[s] = wave_lds[s * P::PS + off];
#pragma unroll
                        for (int s = 0; s < P::FPW; ++s)
                            wave_lds[s * P::PS + off] =
                                make_float2(old[s].x + val[b][s].x, old[s].y + val[b][s].y);
                    }
                    wave_lds_fence();
                }
                // what is left (third or later in a small transform, any collision in a large
                // one) is rare: LDS float atomics, about three cycles per active lane
                if (P::LOG2D <= 9 ? lvl == 2 : (lvl == 1 || lvl == 2)) {
#pragma unroll
                    for (int s = 0; s < P::FPW; ++s) {
                        atomicAdd(&wave_lds[s * P::PS + off].x, val[b][s].x);
                        atomicAdd(&wave_lds[s * P::PS + off].y, val[b][s].y);
                    }
                }
                wave_lds_fence();
            }
        }
        // 2. FPW transforms per wavefront (run() starts with the intra-wavefront fence)
        wave_lds_fence();
        fft.run(my_slot);
        __syncthreads();
        // 3. per-bin separation and recurrence, two time steps per slot, levels ascending
#pragma unroll
        for (int s = 0; s < P::FPW; ++s) {
#pragma unroll
            for (int b = 0; b < BPT; ++b) {
                const int f = tid + NT * b;
                if (f < NB) {
                    const int fi = pad(f), fc = pad((D - f) & (D - 1));
                    float2 p0 = make_float2(1.f, 0.f), p1 = make_float2(1.f, 0.f);
#pragma unroll
                    for (int l = 0; l < M; ++l) {
                        const float2 *Z = lds + ((size_t)l * P::FPW + s) * P::PS;
                        const float2 z = Z[fi], zc = Z[fc];
                        const float2 C0 = make_float2(z.x + zc.x, z.y - zc.y);
                        const float2 C1 = make_float2(z.y + zc.y, zc.x - z.x);
                        const float2 a_old = A[b][l];
                        const float2 a_mid = cfmaf(p0, C0, a_old);
                        A[b][l] = cfmaf(p1, C1, a_mid);
                        p0 = a_old;
                        p1 = a_mid;
                    }
                }
            }
        }
        __syncthreads();
    }

    // Phi_m = Re(FFT(conj Y_m)) / D with Y_m the Hermitian extension of A_m; slot 0 of wavefront m.
#pragma unroll
    for (int b = 0; b < BPT; ++b) {
        const int f = tid + NT * b;
        if (f < NB) {
#pragma unroll
            for (int l = 0; l < M; ++l) {
                float2 *Y = lds + (size_t)l * P::FPW * P::PS;
                const float2 y = A[b][l];
                Y[pad(f)] = make_float2(y.x, -y.y);
                if (f > 0 && f < D / 2) Y[pad(D - f)] = y;
            }
        }
    }
    __syncthreads();
    fft.run(my_slot);
    wave_lds_fence();
    float *row = out + n * ld_out;
    if (tid == 0) row[0] = 1.0f;
    const float invD = 1.0f / (float)D;
    for (int j = lane; j < D; j += 64) row[1 + (int64_t)m * D + j] = wave_lds[pad(j)].x * invD;
}

}  // namespace tuned
}  // namespace rfsf
