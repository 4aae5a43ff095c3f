#include "pt_epilogue.h"
int pt_launch_gemm_mfma(const pt_gemm_args& g, hipStream_t s) { (void)g; (void)s; return 0; }
