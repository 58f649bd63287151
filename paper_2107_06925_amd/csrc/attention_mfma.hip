#include "device.h"
namespace chimera {
bool attention_mfma_supports(const AttnArgs&) { return false; }
int attention_fwd_mfma(const AttnArgs&, void*) { return fail(CHIMERA_EINVAL, "matrix-core attention not built"); }
int attention_bwd_mfma(const AttnArgs&, void*) { return fail(CHIMERA_EINVAL, "matrix-core attention not built"); }
}
