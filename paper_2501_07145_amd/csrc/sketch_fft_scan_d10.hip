// Tuned sketch/FFT/scan kernels for D = 1024.
#define RFSF_LOG2D 10
#include "sketch_fft_scan_inst.inc"
