// Tuned kernel for steps 3-4 with transforms of length 4096 and 8192 (Sec. 3.5, eqs. (cs), (ts_def), (ts_rec)):
// the power-of-two bucket count 4096 and, above all, bucket counts that are no power of two, whose sketches are
// convolved linearly in a transform of nextpow2(M (D - 1) + 1) points and folded modulo D at the end -- the
// paper's own D = 500 and D = 1000 at five levels need 4096 and 8192 points.
//
// A transform of S * 1024 points (S = 4, 8) is split by decimation in time into S interleaved 1024-point
// transforms: wavefront r of a level gathers the buckets = r (mod S) from the level's staging area and runs the
// one-wavefront transform of sketch_fft_scan_tuned.h on them, with no barrier inside; one radix-S pass over
// the S results, done by all threads of the workgroup in LDS,
//     Z[g + 1024 k] = sum_r  w^(r g) E_r[g]  exp(-2 pi i r k / S),   w = exp(-2 pi i / (1024 S)),
// completes the transform in place (the result of k lies where E_k was). Phase 3 is the one of the other
// kernel, a thread owning the bins f = t, t + NT, ...
//
// A workgroup of S * NTR wavefronts per sequence has NTR levels in flight (two, except with a single level);
// the (pair, level) items of the sequence are dealt to them in order, as described for transforms_in_flight()
// in sketch_fft_scan_tuned.h.
//
// Level slot in LDS (float2 units): S sub-slots of 1088 (a padded 1024-point slot each); the staging area lies
// over them from float2 2 on, in coordinate order; float2 0 is the always-zero source of the gather, rewritten
// at the start of every iteration (the gather words address a level slot with 16-bit byte offsets, which reach
// the staging area but not the end of an 8192-point slot).
#pragma once

#include "sketch_fft_scan_tuned.h"

namespace rfsf {
namespace tuned {

constexpr int kWideStageBase = 2;           // first float2 of the staging area in a level slot

__host__ __device__ constexpr int wide_levels_in_flight(int M) { return M == 1 ? 1 : 2; }
__host__ __device__ constexpr int wide_slot_stride(int S, int twoF)
{
    return ((S * Plan<10>::PD > kWideStageBase + staged(twoF) ? S * Plan<10>::PD : kWideStageBase + staged(twoF)) + 1) & ~1;
}
__host__ __device__ constexpr size_t wide_lds_bytes(int S, int M, int F)
{
    return sizeof(float2) * ((size_t)wide_levels_in_flight(M) * wide_slot_stride(S, 2 * F) + Plan<10>::NTWL);
}

template <int LOG2S, int M, int ORDER, int NTR>
__global__ __launch_bounds__(64 * (1 << LOG2S) * NTR) __attribute__((amdgpu_waves_per_eu(4, 4))) void sketch_fft_scan_wide_kernel(
    const float *__restrict__ dphi, const uint32_t *__restrict__ table, int64_t L,
    const int64_t *__restrict__ lengths, int F, int Dout, float *__restrict__ out, int64_t ld_out, TimeCut cut)
{
    using P = Plan<10>;                                     // the transform each wavefront runs
    constexpr int S = 1 << LOG2S, DH = 1024, DF = S * DH, NT = 64 * S * NTR;
    constexpr bool kStream = NTR != M;
    constexpr int BPT = (DF / 2) / NT;                      // bins per thread; thread 0 also carries bin DF/2 (packed)
    static_assert(BPT * NT == DF / 2, "the threads must divide the bins");
    constexpr int BFPT = (NTR * DH) / NT;                   // radix-S butterflies of the combining pass per thread
    static_assert(BFPT * NT == NTR * DH, "the threads must divide the butterflies");
    extern __shared__ float2 lds[];                         // [NTR][PS] level slots, then the twiddle table
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wvl = wave >> LOG2S, res = wave & (S - 1);    // level slot of the workgroup; residue class of the buckets
    const int twoF = 2 * F;
    const int PS = wide_slot_stride(S, twoF);
    float2 *twl_table = lds + (size_t)NTR * PS;
    float2 *lvl_slot = lds + (size_t)wvl * PS;
    char *lvl_bytes = reinterpret_cast<char *>(lvl_slot);
    float2 *sub_slot = lvl_slot + res * P::PD;
    float2 *stage = lvl_slot + kWideStageBase;
    // row of out, sequence, piece of the sequence and the piece's own steps, as in the kernel for shorter transforms
    const int64_t row_id = blockIdx.x;
    const int64_t n = cut.pieces == 1 ? row_id : row_id / cut.pieces, piece = row_id - n * cut.pieces;
    const int64_t Ln = lengths ? (lengths[n] < 1 ? 1 : (lengths[n] > L ? L : lengths[n])) : L;
    const int64_t steps_left = Ln - 1 - 2 * piece * cut.pairs;
    const int64_t T = cut.mode == 2 || steps_left < 0 ? 0 : (steps_left < 2 * cut.pairs ? steps_left : 2 * cut.pairs);
    const int64_t pairs = (T + 1) / 2;
    const int64_t pf = (int64_t)cut.row_levels * 2 * twoF;
    const float *seq = dphi + (n * ((L + 1) / 2) + piece * cut.pairs) * pf;
    const TableLayout tl = table_layout(DF, 64, twoF);
    const int nload = staged(twoF) / 128;
    const float *seq_fixed = seq + (int64_t)wvl * 2 * twoF;
    const uint32_t *tab_fixed = table + (int64_t)wvl * tl.words;

    WaveFft<P> fft;
    fft.init(lane, twl_table);
    __syncthreads();

    float2 A[BPT][M];
#pragma unroll
    for (int b = 0; b < BPT; ++b)
#pragma unroll
        for (int l = 0; l < M; ++l) A[b][l] = make_float2(0.f, 0.f);
    // accumulators kept outside the kernel (sequences cut in time): M levels of bins 0 .. DF/2 per row
    float2 *spectra_row = cut.mode != 0 ? cut.spectra + row_id * (int64_t)(M * (DF / 2 + 1)) : nullptr;
    if (cut.mode == 2) {
#pragma unroll
        for (int b = 0; b < BPT; ++b) {
            const int f = tid + NT * b;
#pragma unroll
            for (int l = 0; l < M; ++l) {
                const float2 *sp = spectra_row + l * (DF / 2 + 1);
                A[b][l] = f == 0 ? make_float2(sp[0].x, sp[DF / 2].x) : sp[f];
            }
        }
    }
    // w^g of the thread's butterflies of the combining pass: butterfly c is number tid + NT * c of the NTR * 1024
    float2 wg[BFPT];
#pragma unroll
    for (int c = 0; c < BFPT; ++c) {
        float s, co;
        sincospif(-(float)((tid + NT * c) & (DH - 1)) * (2.0f / (float)DF), &s, &co);
        wg[c] = make_float2(co, s);
    }
    // Position in a level slot of value f of the complete transform (after the combining pass) and of sample k
    // of its input (before the first pass).
    auto zpos = [](int f) { return (f >> 10) * P::PD + pad(f & (DH - 1)); };
    auto ypos = [](int k) { return (k & (S - 1)) * P::PD + pad(k >> LOG2S); };
    // the radix-S pass over the sub-transforms of every level slot, in place
    auto combine = [&]() {
#pragma unroll
        for (int c = 0; c < BFPT; ++c) {
            const int i = tid + NT * c;
            float2 *base = lds + (size_t)(i >> 10) * PS + pad(i & (DH - 1));
            float2 x[S];
#pragma unroll
            for (int r = 0; r < S; ++r) x[r] = base[r * P::PD];
            // w^(r g), r = 1 .. S-1, from w^g by at most three multiplications each
            float2 wp[S];
            wp[1] = wg[c];
#pragma unroll
            for (int r = 2; r < S; ++r) wp[r] = cmulf(wp[r / 2], wp[r - r / 2]);
#pragma unroll
            for (int r = 1; r < S; ++r) x[r] = cmulf(x[r], wp[r]);
            dft_dif<S, 0, S>(x);
#pragma unroll
            for (int k = 0; k < S; ++k) base[k * P::PD] = x[bitrev(k, LOG2S)];
        }
    };

    auto stage_direct = [&](int lvl, int64_t pair0, int lane_now) {   // the wavefronts of the level take the loads in turn
        const int64_t p = pair0 < pairs ? pair0 : pairs - 1;
        const float *src = (kStream ? seq + (int64_t)lvl * 2 * twoF : seq_fixed) + p * pf + 4 * lane_now;
        for (int j = res; j < nload; j += S)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + 256 * j),
                                             (__attribute__((address_space(3))) void *)(stage + 128 * j), 16, 0, 0);
    };

    int lvl = kStream ? wvl % M : wvl;
    int64_t pair0 = kStream ? wvl / M : 0;
    auto advance = [&](int &l, int64_t &p0) {
        if constexpr (kStream) {
            l += NTR % M;
            p0 += NTR / M;
            if (l >= M) {
                l -= M;
                p0 += 1;
            }
        } else {
            p0 += 1;
        }
    };
    int lvl_first = 0;
    int64_t pair0_first = 0;
    LevelCarry<ORDER> carry[BPT];
    uint32_t gw[P::R], fw[kFoldInRegs];

    __builtin_amdgcn_s_setprio(1);
    // An iteration exists while its first item does. Streaming: the last iteration may have fewer items than
    // level slots; the wavefronts without one run the iteration all the same, on the last pair of their level
    // (stage_direct clamps), and phase 3 ignores what they produce.
    while ((kStream ? pair0_first : pair0) < pairs) {
        // (addresses derived from the lane are recomputed every iteration: hoisted out of the loop they are spilled)
        int lane_here = lane, tid_here = tid;
        asm volatile("" : "+v"(lane_here));
        asm volatile("" : "+v"(tid_here));
        const uint32_t *tabl = kStream ? table + (int64_t)lvl * tl.words : tab_fixed;
        asm volatile("" : "+s"(tabl));
        const GlobalWords tabi = (GlobalWords)tabl;
        int NG = 0;
#pragma unroll
        for (int q = 0; q < P::R; ++q) gw[q] = tabi[tl.gather + S * (lane_here + 64 * q) + res];
        if (res == 0) {
            NG = (int)tabi[0];
#pragma unroll
            for (int g = 0; g < kFoldInRegs; ++g) fw[g] = g < NG ? tabi[tl.fold + g * 64 + lane_here] : kFoldPad << 16;
        }
        stage_direct(lvl, pair0, lane_here);
        __builtin_amdgcn_s_waitcnt(0x0f70);                 // vmcnt(0): this wavefront's direct loads have landed
        if ((T & 1) && pair0 + 1 >= pairs) {                // odd number of increments: the last pair has no second step
            for (int j = res; j < nload; j += S)            // (in the parts this wavefront has loaded itself)
                for (int a = 128 * j + lane_here; a < 128 * j + 128 && a < twoF; a += 64) stage[a].y = 0.f;
        }
        if (res == 0 && lane_here == 0) lvl_slot[0] = make_float2(0.f, 0.f);
        __syncthreads();                                    // the pair is staged
        if (res == 0) {
            auto fold = [&](uint32_t w) {
                const uint32_t own = w & 0xffffu, tgt = w >> 16;
                if (tgt != kFoldPad) {
                    const float2 x = *reinterpret_cast<const float2 *>(lvl_bytes + own);
                    const float2 y = *reinterpret_cast<const float2 *>(lvl_bytes + tgt);
                    *reinterpret_cast<float2 *>(lvl_bytes + tgt) = make_float2(x.x + y.x, x.y + y.y);
                }
                wave_lds_fence();
            };
#pragma unroll
            for (int g = 0; g < kFoldInRegs; ++g)
                if (g < NG) fold(fw[g]);
            for (int g = kFoldInRegs; g < NG; ++g) fold(tabi[tl.fold + g * 64 + lane_here]);
        }
        __syncthreads();                                    // folded
        float2 v[P::R];
#pragma unroll
        for (int q = 0; q < P::R; ++q) {
            const float2 x0 = *reinterpret_cast<const float2 *>(lvl_bytes + (gw[q] & 0xffffu));
            const float2 x1 = *reinterpret_cast<const float2 *>(lvl_bytes + (gw[q] >> 16));
            v[q] = make_float2(x0.x + x1.x, x0.y + x1.y);
            if (q % 4 == 3) __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();                                    // all residues gathered: the staging area may be overwritten
        __builtin_amdgcn_s_setprio(0);
        fft.run_from_registers(sub_slot, v);
        __builtin_amdgcn_s_setprio(1);
        __syncthreads();
        combine();
        __syncthreads();
        // phase 3
        auto update_bin = [&](auto level_tag, auto packed_tag, auto full_tag, int b, int j, int64_t pair0_j) {
            constexpr int LL = decltype(level_tag)::value;
            constexpr bool PK = decltype(packed_tag)::value != 0;
            constexpr bool FULL = decltype(full_tag)::value != 0;
            const int f = tid_here + NT * b;
            const bool pk = PK && b == 0 && f == 0;
            const bool second_step = FULL || 2 * pair0_j + 1 < T;
            const float2 *Z = lds + (size_t)j * PS;
            const float2 z = Z[zpos(f)], zc = Z[zpos(f > 0 ? DF - f : DF / 2)];
            level_step<ORDER, LL, PK>(z, zc, pk, second_step, A[b][LL], carry[b]);
        };
        auto phase3 = [&](auto packed_tag, auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value != 0;
            if constexpr (kStream) {
                with_level<M>(lvl_first, [&](auto first_tag) {
                    constexpr int L0 = decltype(first_tag)::value;
                    item_loop<L0, M, NTR>([&](auto level_tag, auto item_tag, int group_offset) {
                        constexpr int j = decltype(item_tag)::value;
                        const int64_t pair0_j = pair0_first + group_offset;
                        if (FULL || pair0_j < pairs) {
#pragma unroll
                            for (int b = 0; b < BPT; ++b) update_bin(level_tag, packed_tag, full_tag, b, j, pair0_j);
                        }
                    });
                });
            } else {
                level_loop<M>([&](auto level_tag) {
#pragma unroll
                    for (int b = 0; b < BPT; ++b)
                        update_bin(level_tag, packed_tag, full_tag, b, decltype(level_tag)::value, pair0);
                });
            }
        };
        const int64_t last_pair0 = kStream ? pair0_first + (lvl_first + NTR - 1) / M : pair0;
        const bool full = 2 * (last_pair0 + 1) - 1 < T;
        if (wave == 0) {
            if (full) phase3(LevelTag<1>{}, LevelTag<1>{});
            else phase3(LevelTag<1>{}, LevelTag<0>{});
        } else {
            if (full) phase3(LevelTag<0>{}, LevelTag<1>{});
            else phase3(LevelTag<0>{}, LevelTag<0>{});
        }
        advance(lvl, pair0);
        if constexpr (kStream) advance(lvl_first, pair0_first);
        __syncthreads();                                    // the slots are free again
    }

    if (cut.mode == 1) {                                    // a piece of a sequence: its accumulators are the result
#pragma unroll
        for (int b = 0; b < BPT; ++b) {
            const int f = tid + NT * b;
#pragma unroll
            for (int l = 0; l < M; ++l) {
                float2 *sp = spectra_row + l * (DF / 2 + 1);
                const float2 a = A[b][l];
                if (f == 0) {                               // bins 0 and DF/2 are real
                    sp[0] = make_float2(a.x, 0.f);
                    sp[DF / 2] = make_float2(a.y, 0.f);
                } else {
                    sp[f] = a;
                }
            }
        }
        return;
    }

    // Phi_l = Re(FFT(conj Y_l)) / DF with Y_l the Hermitian extension of A_l, NTR levels at a time
    float *row = out + row_id * ld_out;
    if (tid == 0) row[0] = 1.0f;
#pragma unroll
    for (int l0 = 0; l0 < M; l0 += NTR) {
#pragma unroll
        for (int j = 0; j < NTR; ++j) {
            if (l0 + j < M) {
                float2 *base = lds + (size_t)j * PS;
#pragma unroll
                for (int b = 0; b < BPT; ++b) {
                    const int f = tid + NT * b;
                    const float2 a = A[b][l0 + j < M ? l0 + j : 0];
                    if (f == 0) {                           // bins 0 and DF/2 are real
                        base[ypos(0)] = make_float2(a.x, 0.f);
                        base[ypos(DF / 2)] = make_float2(a.y, 0.f);
                    } else {
                        base[ypos(f)] = make_float2(a.x, -a.y);
                        base[ypos(DF - f)] = a;
                    }
                }
            }
        }
        __syncthreads();
        const bool mine = l0 + wvl < M;
        if (mine) fft.run(sub_slot);
        __syncthreads();
        combine();
        __syncthreads();
        if (mine) {
            const float invD = 1.0f / (float)DF;
            for (int j = res * 64 + lane; j < Dout; j += 64 * S) {
                float acc = 0.f;
                for (int e = j; e < DF; e += Dout) acc += lvl_slot[zpos(e)].x;
                row[1 + (int64_t)(l0 + wvl) * Dout + j] = acc * invD;
            }
        }
        if (l0 + NTR < M) __syncthreads();
    }
}

template <int LOG2S, int M, int ORDER>
hipError_t launch_wide(const float *dphi, const uint32_t *table, int64_t n_seq, int64_t L, const int64_t *lengths, int F, int Dout,
                       float *out, int64_t ld_out, hipStream_t stream, TimeCut cut)
{
    constexpr int S = 1 << LOG2S, NTR = wide_levels_in_flight(M);
    const size_t lds = wide_lds_bytes(S, M, F);
    auto kernel = sketch_fft_scan_wide_kernel<LOG2S, M, ORDER, NTR>;
    if (lds > 64 * 1024) {
        static size_t raised = 0;
        if (lds > raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            raised = lds;
        }
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)(n_seq * cut.pieces)), dim3(64 * S * NTR), lds, stream, dphi, table, L, lengths, F, Dout, out, ld_out, cut);
    return hipGetLastError();
}

template <int LOG2S>
hipError_t dispatch_wide(int M, int order, const float *dphi, const uint32_t *table, int64_t n_seq, int64_t L, const int64_t *lengths,
                         int F, int Dout, float *out, int64_t ld_out, hipStream_t stream, TimeCut cut)
{
    switch (M) {
#define RFSF_CASE(MM)                                                                                                  \
        case MM:                                                                                                       \
            return order == 3 ? launch_wide<LOG2S, MM, 3>(dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut)    \
                 : order == 2 ? launch_wide<LOG2S, MM, 2>(dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut)    \
                              : launch_wide<LOG2S, MM, 1>(dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
        RFSF_CASE(1) RFSF_CASE(2) RFSF_CASE(3) RFSF_CASE(4) RFSF_CASE(5) RFSF_CASE(6) RFSF_CASE(7) RFSF_CASE(8)
#undef RFSF_CASE
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tuned
}  // namespace rfsf
