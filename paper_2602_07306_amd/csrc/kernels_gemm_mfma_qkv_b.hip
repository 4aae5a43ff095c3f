// MFMA GEMM kernels with the EPI_QKV epilogue, tile configurations 1, 4, 8 (the heaviest epilogue to compile:
// its configurations are spread over four translation units).
#include "gemm_mfma_impl.h"

PT_GEMM_INSTANTIATE(EPI_QKV, 1)
PT_GEMM_INSTANTIATE(EPI_QKV, 4)
PT_GEMM_INSTANTIATE(EPI_QKV, 8)
