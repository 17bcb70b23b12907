// Group sweep / commit kernels of the BPDQ pass for k = 4 bit-planes (all group sizes).
#include "group_sweep.h"

namespace bpdq {
GroupLauncher pick_group_k4(int g) { return pick_group_g<4>(g); }
}  // namespace bpdq
