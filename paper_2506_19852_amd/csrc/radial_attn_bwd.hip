// Block-sparse attention backward (placeholder until the kernels land: fails loudly).
#include "radial_internal.h"

namespace radial {
int launch_bwd(int, int, const BwdArgs&, hipStream_t) {
  return fail(RADIAL_EUNSUPPORTED, "radial_attn_bwd is not implemented yet");
}
}  // namespace radial
