// Instantiations of the fused transform core on the min/max grid of Eq. (1) for 32 x 32 transform blocks.
#include "xform_launch.hpp"
namespace cafeq {
int launch_core_asym_k32(int G, int axis, const CoreParams& p, hipStream_t st) { return launch_core_asym_k<32>(G, axis, p, st); }
}  // namespace cafeq
