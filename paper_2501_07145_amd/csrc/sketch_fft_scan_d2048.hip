// Tuned sketch/FFT/scan kernels for transforms of 2048 points held by one wavefront (Plan<2048>).
#define RFSF_LOG2D 2048
#include "sketch_fft_scan_inst.inc"
