// MFMA GEMM kernels with the EPI_QKV epilogue, tile configurations 0, 10, 11 (the heaviest epilogue to compile:
// its configurations are spread over four translation units).
#include "gemm_mfma_impl.h"

PT_GEMM_INSTANTIATE(EPI_QKV, 0)
PT_GEMM_INSTANTIATE(EPI_QKV, 10)
PT_GEMM_INSTANTIATE(EPI_QKV, 11)
