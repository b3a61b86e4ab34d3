// Instantiates the fused attention-layer kernel for inputs that occupy 6 slots of 64 floats.
#include "layer_kernel.h"

namespace stgn {
template void layer_entry<6>(layer_impl::LaunchArgs&);
}  // namespace stgn
