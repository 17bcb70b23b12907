// Group sweep / commit kernels of the BPDQ pass for k = 1 bit-plane (all group sizes).
#include "group_sweep.h"

namespace bpdq {
GroupLauncher pick_group_k1(int g) { return pick_group_g<1>(g); }
}  // namespace bpdq
