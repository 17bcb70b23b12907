// Group sweep / commit kernels of the BPDQ pass for k = 4, group size 256.
#include "group_sweep.h"

namespace bpdq {
GroupLauncher group256_k4() { return launch_group<4, 256>; }
}  // namespace bpdq
