// Fixed-uniform-grid sweep kernel of the BPDQ pass for k = 1, group size 256.
#include "group_sweep.h"

namespace bpdq {
template <>
int launch_uniform_sweep_256<1>(const UniformSweepArgs& a) { return launch_uniform_sweep<1, 256>(a); }
}  // namespace bpdq
