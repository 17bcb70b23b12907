// Fixed-uniform-grid sweep kernel of the BPDQ pass for k = 3, group size 256.
#include "group_sweep.h"

namespace bpdq {
template <>
int launch_uniform_sweep_256<3>(const UniformSweepArgs& a) { return launch_uniform_sweep<3, 256>(a); }
}  // namespace bpdq
