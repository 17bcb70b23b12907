// Group sweep / commit kernels of the BPDQ pass for k = 1, group size 256.
#include "group_sweep.h"

namespace bpdq {
GroupLauncher group256_k1() { return launch_group<1, 256>; }
}  // namespace bpdq
