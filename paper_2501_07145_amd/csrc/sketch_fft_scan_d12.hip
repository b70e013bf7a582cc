// Tuned sketch/FFT/scan kernels for transforms of 4096 points.
#include "sketch_fft_scan_dispatch.h"
#include "sketch_fft_scan_wide.h"

namespace rfsf {
namespace tuned {

hipError_t dispatch_levels_12(int M, int order, const float *dphi, const uint32_t *table, int64_t n_seq, int64_t L,
                              const int64_t *lengths, int F, int Dout, float *out, int64_t ld_out, hipStream_t stream,
                              TimeCut cut)
{
    return dispatch_wide<2>(M, order, dphi, table, n_seq, L, lengths, F, Dout, out, ld_out, stream, cut);
}

}  // namespace tuned
}  // namespace rfsf
