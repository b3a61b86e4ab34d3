// Instantiates the fused attention-layer kernel for 4 attention head(s).
#include "layer_kernel.h"

namespace stgn {
template void layer_entry<4>(layer_impl::LaunchArgs&);
}  // namespace stgn
