// Instantiates the fused attention-layer kernel for 1 attention head(s).
#include "layer_kernel.h"

namespace stgn {
template void layer_entry<1>(layer_impl::LaunchArgs&);
}  // namespace stgn
