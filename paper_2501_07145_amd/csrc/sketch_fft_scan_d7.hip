// Tuned sketch/FFT/scan kernels for D = 128.
#define RFSF_LOG2D 7
#include "sketch_fft_scan_inst.inc"
