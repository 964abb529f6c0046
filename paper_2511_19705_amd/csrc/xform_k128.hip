// Instantiations of the fused transform core for 128 x 128 transform blocks.
#include "xform_launch.hpp"
#include "grad_core.hpp"
namespace cafeq {
int launch_core_k128(int G, int axis, const CoreParams& p, hipStream_t st) { return launch_core_k<128>(G, axis, p, st); }
size_t core_lds_bytes_k128(int G, bool do_grad) { return core_lds_bytes_k<128>(G, do_grad); }

namespace {
template <int G, int AXIS>
int launch_grad_t(const CoreParams& p, hipStream_t st) {
  using g = Geo<128, G>;
  constexpr size_t lds = size_t(g::GRADB) + 64;
  auto kern = grad_z_kernel<128, G, AXIS>;
  static bool attr_set = false;   // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            int(kMaxLds)) != hipSuccess)
      return CAFEQ_ERR_LAUNCH;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(unsigned(p.nwg)), dim3(kThreads), lds, st, p);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
}  // namespace

int launch_grad_k128(int G, int axis, const CoreParams& p, hipStream_t st) {
  const bool col = axis == CAFEQ_AXIS_COL;
  switch (G) {
    case 32: return col ? launch_grad_t<32, CAFEQ_AXIS_COL>(p, st) : launch_grad_t<32, CAFEQ_AXIS_ROW>(p, st);
    case 64: return col ? launch_grad_t<64, CAFEQ_AXIS_COL>(p, st) : launch_grad_t<64, CAFEQ_AXIS_ROW>(p, st);
    case 128: return col ? launch_grad_t<128, CAFEQ_AXIS_COL>(p, st) : launch_grad_t<128, CAFEQ_AXIS_ROW>(p, st);
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
}
}  // namespace cafeq
