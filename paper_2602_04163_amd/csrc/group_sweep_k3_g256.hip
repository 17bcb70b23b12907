// Group sweep / commit kernels of the BPDQ pass for k = 3, group size 256.
#include "group_sweep.h"

namespace bpdq {
GroupLauncher group256_k3() { return launch_group<3, 256>; }
}  // namespace bpdq
