// MFMA GEMM kernels with the EPI_QKV epilogue, tile configurations 5, 6, 7 (the heaviest epilogue to compile:
// its configurations are spread over four translation units).
#include "gemm_mfma_impl.h"

PT_GEMM_INSTANTIATE(EPI_QKV, 5)
PT_GEMM_INSTANTIATE(EPI_QKV, 6)
PT_GEMM_INSTANTIATE(EPI_QKV, 7)
