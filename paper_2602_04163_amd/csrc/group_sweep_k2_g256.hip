// Group sweep / commit kernels of the BPDQ pass for k = 2, group size 256.
#include "group_sweep.h"

namespace bpdq {
GroupLauncher group256_k2() { return launch_group<2, 256>; }
}  // namespace bpdq
