#include "device.h"
namespace chimera {
bool gemm_mfma_supports(const GemmArgs&) { return false; }
int gemm_mfma_bf16(const GemmArgs&, void*) { return fail(CHIMERA_EINVAL, "matrix-core gemm not built"); }
}
