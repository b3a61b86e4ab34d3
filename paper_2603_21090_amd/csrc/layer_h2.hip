// Instantiates the fused attention-layer kernel for 2 attention head(s).
#include "layer_kernel.h"

namespace stgn {
template void layer_entry<2>(layer_impl::LaunchArgs&);
}  // namespace stgn
