// Instantiations and launchers of the gradient pass of the two-pass scheme (grad_core.hpp).
#include "xform_launch.hpp"
#include "grad_core.hpp"
namespace cafeq {

namespace {
template <int K, int AXIS>
int launch_grad_t(const CoreParams& p, hipStream_t st) {
  using g = GradGeo<K>;
  constexpr size_t lds = size_t(g::LDSB);
  static_assert((K == 256 ? 1 : 2) * lds <= kMaxLds, "workgroups per compute unit");
  auto kern = grad_z_kernel<K, AXIS>;
  static std::atomic<bool> attr_set{false};   // per instantiation
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

size_t grad_pass_part_floats(int K) {
  switch (K) {
    case 32: return GradGeo<32>::PART;
    case 64: return GradGeo<64>::PART;
    case 128: return GradGeo<128>::PART;
    case 256: return GradGeo<256>::PART;
    default: return 0;
  }
}

int launch_grad_pass(int K, int axis, const CoreParams& p, hipStream_t st) {
  const bool col = axis == CAFEQ_AXIS_COL;
  if (!p.rec || !p.slot_grad || p.grp < 32 || p.grp % 32 != 0) return CAFEQ_ERR_INVALID_ARG;
  switch (K) {
    case 32: return col ? launch_grad_t<32, CAFEQ_AXIS_COL>(p, st) : launch_grad_t<32, CAFEQ_AXIS_ROW>(p, st);
    case 64: return col ? launch_grad_t<64, CAFEQ_AXIS_COL>(p, st) : launch_grad_t<64, CAFEQ_AXIS_ROW>(p, st);
    case 128: return col ? launch_grad_t<128, CAFEQ_AXIS_COL>(p, st) : launch_grad_t<128, CAFEQ_AXIS_ROW>(p, st);
    case 256: return col ? launch_grad_t<256, CAFEQ_AXIS_COL>(p, st) : launch_grad_t<256, CAFEQ_AXIS_ROW>(p, st);
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
}

int launch_combine_records(const float2* rec, int gspan, int L, int64_t nlines, int64_t ngroups, float2* grec,
                           hipStream_t st, const float2* rec_mm, float2* grec_mm) {
  const int64_t n = ngroups * nlines;
  hipLaunchKernelGGL(combine_records_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, rec, gspan, L, nlines,
                     ngroups, grec, rec_mm, grec_mm);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

}  // namespace cafeq
