// Instantiations of the fused transform core for 64 x 64 transform blocks.
#include "xform_launch.hpp"
namespace cafeq {
int launch_core_k64(int G, int axis, const CoreParams& p, hipStream_t st) { return launch_core_k<64>(G, axis, p, st); }
size_t core_lds_bytes_k64(int G, bool do_grad) { return core_lds_bytes_k<64>(G, do_grad); }
}  // namespace cafeq
