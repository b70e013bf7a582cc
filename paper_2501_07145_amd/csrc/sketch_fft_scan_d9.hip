// Tuned sketch/FFT/scan kernels for D = 512.
#define RFSF_LOG2D 9
#include "sketch_fft_scan_inst.inc"
