// bf16 MFMA GEMM / implicit-GEMM convolution (placeholder until the MFMA kernels land).
#include "kernels.h"
namespace pserve {
int gemm_mfma_bf16(const GemmArgs& a, hipStream_t st, bool* handled) { (void)a; (void)st; *handled = false; return PSERVE_OK; }
}
