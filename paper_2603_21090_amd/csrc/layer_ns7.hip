// Instantiates the fused attention-layer kernel for inputs that occupy 7 slots of 64 floats.
#include "layer_kernel.h"

namespace stgn {
template void layer_entry<7>(layer_impl::LaunchArgs&);
}  // namespace stgn
