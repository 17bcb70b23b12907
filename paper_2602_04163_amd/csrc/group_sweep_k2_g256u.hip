// Fixed-uniform-grid sweep kernel of the BPDQ pass for k = 2, group size 256.
#include "group_sweep.h"

namespace bpdq {
template <>
int launch_uniform_sweep_256<2>(const UniformSweepArgs& a) { return launch_uniform_sweep<2, 256>(a); }
}  // namespace bpdq
