// Tuned sketch/FFT/scan kernels for exact transforms of 200 points (Plan<200>).
#define RFSF_LOG2D 200
#include "sketch_fft_scan_inst.inc"
