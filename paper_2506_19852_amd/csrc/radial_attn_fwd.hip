// Forward entry of the library: the kernel template of radial_attn_fwd_kernel.h without trace records.
#include "radial_attn_fwd_kernel.h"

namespace radial {

int64_t fwd_grid(const FwdArgs& a) { return 8LL * a.B * a.H * a.max_slice; }

int launch_fwd(int D, int block, const FwdArgs& a, hipStream_t stream) { return fwd::launch_any<false>(D, block, a, stream); }

}  // namespace radial
