// Tuned sketch/FFT/scan kernels for D = 64.
#define RFSF_LOG2D 6
#include "sketch_fft_scan_inst.inc"
