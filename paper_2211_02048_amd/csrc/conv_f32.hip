// The convolution kernels for storage type float: this translation unit instantiates them (one per type, so
// that the three compile side by side).
#include "conv_kernels.h"

namespace sige {
SIGE_CONV_LAUNCHERS(, float)
}  // namespace sige
