// Tuned sketch/FFT/scan kernels for exact transforms of 500 points (Plan<500>).
#define RFSF_LOG2D 500
#include "sketch_fft_scan_inst.inc"
