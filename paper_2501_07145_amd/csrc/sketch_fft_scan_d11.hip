// Tuned sketch/FFT/scan kernels for D = 2048.
#define RFSF_LOG2D 11
#include "sketch_fft_scan_inst.inc"
