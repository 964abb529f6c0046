// Instantiations of the fused transform core for 128 x 128 transform blocks.
#include "xform_launch.hpp"
namespace cafeq {
int launch_core_k128(int G, int axis, const CoreParams& p, hipStream_t st) { return launch_core_k<128>(G, axis, p, st); }
size_t core_lds_bytes_k128(int G, bool do_grad) { return core_lds_bytes_k<128>(G, do_grad); }
}  // namespace cafeq
