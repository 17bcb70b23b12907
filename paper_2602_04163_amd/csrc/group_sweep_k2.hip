// Group sweep / commit kernels of the BPDQ pass for k = 2 bit-planes (all group sizes).
#include "group_sweep.h"

namespace bpdq {
GroupLauncher pick_group_k2(int g) { return pick_group_g<2>(g); }
}  // namespace bpdq
