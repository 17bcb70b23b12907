// Group sweep / commit kernels of the BPDQ pass for k = 3 bit-planes (all group sizes).
#include "group_sweep.h"

namespace bpdq {
GroupLauncher pick_group_k3(int g) { return pick_group_g<3>(g); }
}  // namespace bpdq
