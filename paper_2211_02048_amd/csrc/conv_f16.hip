// The convolution kernels for storage type f16: this translation unit instantiates them (one per type, so
// that the three compile side by side).
#include "conv_kernels.h"

namespace sige {
SIGE_CONV_LAUNCHERS(, f16)
}  // namespace sige
