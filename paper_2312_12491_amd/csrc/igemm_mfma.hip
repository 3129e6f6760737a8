// bf16 MFMA implicit GEMM (placeholder until the kernel lands: nothing is routed here).
#include "common.h"
bool igemm_mfma_available() { return false; }
bool igemm_mfma_supported(const IgemmParams&) { return false; }
void launch_igemm_mfma(const IgemmParams&, hipStream_t) {}
