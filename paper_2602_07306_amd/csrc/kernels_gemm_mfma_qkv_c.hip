// MFMA GEMM kernels with the EPI_QKV epilogue, tile configurations 2, 3, 9 (the heaviest epilogue to compile:
// its configurations are spread over four translation units).
#include "gemm_mfma_impl.h"

PT_GEMM_INSTANTIATE(EPI_QKV, 2)
PT_GEMM_INSTANTIATE(EPI_QKV, 3)
PT_GEMM_INSTANTIATE(EPI_QKV, 9)
