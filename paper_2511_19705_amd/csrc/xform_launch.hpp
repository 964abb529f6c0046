// Host launcher template for the fused core; included by the per-K instantiation files.
#pragma once
#include "xform_core.hpp"

namespace cafeq {

constexpr size_t kMaxLds = 160 * 1024;

// LDS bytes of one workgroup; 0 means "the gradient is not available for this (K, G)".
template <int K, int G>
constexpr size_t core_lds_bytes_t(bool do_grad) {
  using g = Geo<K, G>;
  if (do_grad && !g::GRAD_OK) return 0;
  return size_t(g::RINGB) + (do_grad ? size_t(g::GRADB) : 0) + size_t(g::MISCB);
}

// The half-precision forward variant exists for 128 x 128 blocks with one block per segment.
template <int K, int G>
constexpr bool core_has_f16() { return K == 128 && Geo<K, G>::NBLK == 1; }

template <int K, int G, int AXIS, bool GRAD, bool F16 = false, bool LONGG = false, bool ASYM = false>
int launch_core_v(const CoreParams& p, size_t lds, hipStream_t st) {
  auto kern = xform_core_kernel<K, G, AXIS, GRAD, F16, LONGG, ASYM>;
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

template <int K, int G, int AXIS>
int launch_core_t(const CoreParams& p, hipStream_t st) {
  const size_t lds = core_lds_bytes_t<K, G>(p.do_grad != 0);
  if (lds == 0 || lds > kMaxLds) return CAFEQ_ERR_UNSUPPORTED;
  // half-precision forward planes (p.fscale set): only for the gradient-free variant, where it exists
  if (p.fscale && (p.do_grad || !core_has_f16<K, G>())) return CAFEQ_ERR_INVALID_ARG;
  // groups that span several segments: the segment is one group of max(K, 128) (or K) elements
  if (p.longg) {
    if constexpr (G >= K && (G == K || G == 128)) {
      if (p.do_grad) return CAFEQ_ERR_INVALID_ARG;
      if constexpr (core_has_f16<K, G>()) {
        if (p.fscale) return launch_core_v<K, G, AXIS, false, true, true>(p, lds, st);
      }
      return launch_core_v<K, G, AXIS, false, false, true>(p, lds, st);
    } else {
      return CAFEQ_ERR_UNSUPPORTED;
    }
  }
  if constexpr (Geo<K, G>::GRAD_OK) {
    if (p.do_grad) return launch_core_v<K, G, AXIS, true>(p, lds, st);
  }
  if constexpr (core_has_f16<K, G>()) {
    if (p.fscale) return launch_core_v<K, G, AXIS, false, true>(p, lds, st);
  }
  return launch_core_v<K, G, AXIS, false>(p, lds, st);
}

template <int K>
int launch_core_k(int G, int axis, const CoreParams& p, hipStream_t st) {
#define CAFEQ_CORE_CASE(GG)                                                           \
  case GG:                                                                            \
    return axis == CAFEQ_AXIS_COL ? launch_core_t<K, GG, CAFEQ_AXIS_COL>(p, st)       \
                                  : launch_core_t<K, GG, CAFEQ_AXIS_ROW>(p, st);
  switch (G) {
    CAFEQ_CORE_CASE(32)
    CAFEQ_CORE_CASE(64)
    CAFEQ_CORE_CASE(128)
    CAFEQ_CORE_CASE(256)
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
#undef CAFEQ_CORE_CASE
}

// The variants for the min/max grid of Eq. (1) (instantiated in translation units of their own): gradient-free,
// full-precision forward, with and without groups that span segments.
template <int K, int G, int AXIS>
int launch_core_asym_t(const CoreParams& p, hipStream_t st) {
  const size_t lds = core_lds_bytes_t<K, G>(false);
  if (lds == 0 || lds > kMaxLds) return CAFEQ_ERR_UNSUPPORTED;
  if (p.do_grad || p.fscale) return CAFEQ_ERR_INVALID_ARG;
  if (p.longg) {
    if constexpr (G >= K && (G == K || G == 128)) {
      return launch_core_v<K, G, AXIS, false, false, true, true>(p, lds, st);
    } else {
      return CAFEQ_ERR_UNSUPPORTED;
    }
  }
  return launch_core_v<K, G, AXIS, false, false, false, true>(p, lds, st);
}

template <int K>
int launch_core_asym_k(int G, int axis, const CoreParams& p, hipStream_t st) {
#define CAFEQ_CORE_CASE(GG)                                                                \
  case GG:                                                                                 \
    return axis == CAFEQ_AXIS_COL ? launch_core_asym_t<K, GG, CAFEQ_AXIS_COL>(p, st)       \
                                  : launch_core_asym_t<K, GG, CAFEQ_AXIS_ROW>(p, st);
  switch (G) {
    CAFEQ_CORE_CASE(32)
    CAFEQ_CORE_CASE(64)
    CAFEQ_CORE_CASE(128)
    CAFEQ_CORE_CASE(256)
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
#undef CAFEQ_CORE_CASE
}

template <int K>
size_t core_lds_bytes_k(int G, bool do_grad) {
  switch (G) {
    case 32: return core_lds_bytes_t<K, 32>(do_grad);
    case 64: return core_lds_bytes_t<K, 64>(do_grad);
    case 128: return core_lds_bytes_t<K, 128>(do_grad);
    case 256: return core_lds_bytes_t<K, 256>(do_grad);
    default: return 0;
  }
}

}  // namespace cafeq
