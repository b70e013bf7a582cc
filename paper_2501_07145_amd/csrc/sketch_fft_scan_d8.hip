// Tuned sketch/FFT/scan kernels for D = 256.
#define RFSF_LOG2D 8
#include "sketch_fft_scan_inst.inc"
