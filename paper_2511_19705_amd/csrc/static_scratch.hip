// cafeq_rtn_quantize_static: the plain per-group quantizer for callers that cannot allocate device
// memory or bring a workspace (code under HIP graph capture, tight serving loops).  The only scratch the
// quantizer needs -- one float64 squared-error partial per workgroup -- lives in a file-scope device
// array instead of the caller's `ws`.  See include/cafeq.h.
#include <mutex>

#include "cafeq_internal.hpp"

namespace {

constexpr size_t kMaxPartials = 65536;   // float64 partials: 512 KB per GPU, held until the process ends
static __device__ __align__(256) double scratch[kMaxPartials];

// In host code `scratch` is only a handle for the runtime: the memory's device address is looked up once
// per device (every GPU holds its own copy of the array) and kept.
constexpr int kMaxDevices = 64;
double* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

int scratch_for_current_device(double** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CAFEQ_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CAFEQ_ERR_LAUNCH;
    g_scratch_ptr[dev] = static_cast<double*>(p);
  }
  *out = g_scratch_ptr[dev];
  return CAFEQ_OK;
}

}  // namespace

extern "C" int cafeq_rtn_quantize_static(const cafeq_mat* W, const cafeq_quant_cfg* cfg, int8_t* codes,
                                          float* scales, float* err_sq, void* stream) {
  using namespace cafeq;
  if (!W || !W->data || !cfg || !codes) return CAFEQ_ERR_INVALID_ARG;
  if (W->dtype != CAFEQ_F32 && W->dtype != CAFEQ_BF16) return CAFEQ_ERR_INVALID_ARG;
  if (cfg->bits < 2 || cfg->bits > 8 || cfg->group < 0) return CAFEQ_ERR_INVALID_ARG;
  if (cfg->axis != CAFEQ_AXIS_COL && cfg->axis != CAFEQ_AXIS_ROW) return CAFEQ_ERR_INVALID_ARG;
  if (cfg->mode == CAFEQ_Q_ASYM_MINMAX) return CAFEQ_ERR_UNSUPPORTED;
  if (cfg->mode != CAFEQ_Q_SYM_ABSMAX) return CAFEQ_ERR_INVALID_ARG;
  if (W->rows <= 0 || W->cols <= 0 || W->ld < W->cols || W->cols % 4 != 0) return CAFEQ_ERR_BAD_SHAPE;
  const int64_t ldm = W->dtype == CAFEQ_F32 ? 4 : 8;
  auto misaligned = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
  if (W->ld % ldm != 0 || misaligned(W->data) || misaligned(codes) || (scales && misaligned(scales)))
    return CAFEQ_ERR_BAD_ALIGN;
  const int64_t line = cfg->axis == CAFEQ_AXIS_COL ? W->cols : W->rows;
  const int64_t g = cfg->group == 0 ? line : cfg->group;
  if (line % g != 0) return CAFEQ_ERR_BAD_SHAPE;
  // the size limit of the built-in scratch: one partial per workgroup of whichever kernel is picked
  if (err_sq && rtn_partials_capacity(W->rows, W->cols) > kMaxPartials) return CAFEQ_ERR_WORKSPACE;
  double* partial = nullptr;
  if (err_sq) {
    const int rc = scratch_for_current_device(&partial);
    if (rc) return rc;
  }
  RtnArgs a;
  a.W = W->data; a.dtype = W->dtype; a.rows = W->rows; a.cols = W->cols; a.ld = W->ld;
  a.axis = cfg->axis; a.group = cfg->group; a.grid = make_grid(cfg->bits);
  a.codes = codes; a.scales = scales; a.mins = nullptr;
  a.partial = partial;   // every workgroup overwrites its own partial before the sum reads them: nothing to clear
  a.err_sq = err_sq;
  return launch_rtn(a, static_cast<hipStream_t>(stream));
}
