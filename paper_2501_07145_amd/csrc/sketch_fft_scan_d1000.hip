// Tuned sketch/FFT/scan kernels for exact transforms of 1000 points (Plan<1000>).
#define RFSF_LOG2D 1000
#include "sketch_fft_scan_inst.inc"
