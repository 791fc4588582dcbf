// bf16 MFMA attention (placeholder until the MFMA kernels land).
#include "kernels.h"
namespace pserve {
int attention_mfma_bf16(const AttnArgs& a, hipStream_t st, bool* handled) { (void)a; (void)st; *handled = false; return PSERVE_OK; }
}
