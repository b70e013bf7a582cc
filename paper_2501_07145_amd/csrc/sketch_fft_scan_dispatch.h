// Host-side launch of the tuned sketch/FFT/scan kernel. The instantiations for one transform
// length live in one translation unit each (sketch_fft_scan_d<log2 D>.hip) so that they
// compile in parallel; this header declares their entry points and holds the shared template.
#pragma once

#include "rfsf_internal.h"

namespace rfsf {
namespace tuned {

#define RFSF_DECLARE_DISPATCH(LOG2D)                                                                       \
    hipError_t dispatch_levels_##LOG2D(int M, int order, const float *dphi, const uint32_t *table, int64_t n_seq,     \
                                       int64_t L, const int64_t *lengths, int F, int Dout, float *out, int64_t ld_out, hipStream_t stream, TimeCut cut);
RFSF_DECLARE_DISPATCH(6)
RFSF_DECLARE_DISPATCH(7)
RFSF_DECLARE_DISPATCH(8)
RFSF_DECLARE_DISPATCH(9)
RFSF_DECLARE_DISPATCH(10)
RFSF_DECLARE_DISPATCH(12)
RFSF_DECLARE_DISPATCH(13)
RFSF_DECLARE_DISPATCH(100)
RFSF_DECLARE_DISPATCH(200)
RFSF_DECLARE_DISPATCH(500)
RFSF_DECLARE_DISPATCH(1000)
RFSF_DECLARE_DISPATCH(2048)
#undef RFSF_DECLARE_DISPATCH

}  // namespace tuned
}  // namespace rfsf
