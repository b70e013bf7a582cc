// Tuned sketch/FFT/scan kernels for exact transforms of 100 points (Plan<100>).
#define RFSF_LOG2D 100
#include "sketch_fft_scan_inst.inc"
