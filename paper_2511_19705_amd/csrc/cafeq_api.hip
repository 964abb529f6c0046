// extern "C" entry points: argument validation and dispatch.  See include/cafeq.h.
#include "cafeq_internal.hpp"

using namespace cafeq;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_mat(const cafeq_mat* m) {
  if (!m || !m->data) return CAFEQ_ERR_INVALID_ARG;
  if (m->dtype != CAFEQ_F32 && m->dtype != CAFEQ_BF16) return CAFEQ_ERR_INVALID_ARG;
  if (m->rows <= 0 || m->cols <= 0 || m->ld < m->cols) return CAFEQ_ERR_BAD_SHAPE;
  if (m->cols % 4 != 0) return CAFEQ_ERR_BAD_SHAPE;
  const int64_t ldm = m->dtype == CAFEQ_F32 ? 4 : 8;
  if (m->ld % ldm != 0 || !aligned16(m->data)) return CAFEQ_ERR_BAD_ALIGN;
  return CAFEQ_OK;
}

int check_cfg(const cafeq_quant_cfg* c, bool need_axis) {
  if (!c) return CAFEQ_ERR_INVALID_ARG;
  if (c->bits < 2 || c->bits > 8 || c->group < 0) return CAFEQ_ERR_INVALID_ARG;
  if (need_axis && c->axis != CAFEQ_AXIS_COL && c->axis != CAFEQ_AXIS_ROW) return CAFEQ_ERR_INVALID_ARG;
  if (c->mode == CAFEQ_Q_ASYM_MINMAX) return CAFEQ_ERR_UNSUPPORTED;
  if (c->mode != CAFEQ_Q_SYM_ABSMAX) return CAFEQ_ERR_INVALID_ARG;
  return CAFEQ_OK;
}

}  // namespace

extern "C" {

const char* cafeq_strerror(int status) {
  switch (status) {
    case CAFEQ_OK: return "ok";
    case CAFEQ_ERR_INVALID_ARG: return "invalid argument";
    case CAFEQ_ERR_BAD_SHAPE: return "shape not divisible as required";
    case CAFEQ_ERR_BAD_ALIGN: return "pointer or leading dimension misaligned";
    case CAFEQ_ERR_UNSUPPORTED: return "configuration not supported by this build";
    case CAFEQ_ERR_SINGULAR: return "singular transform block";
    case CAFEQ_ERR_LAUNCH: return "HIP launch failed";
    case CAFEQ_ERR_WORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
  }
}

int cafeq_version(void) { return 100; }

size_t cafeq_workspace_bytes(int call_id, const cafeq_mat* a, const cafeq_mat* b, const cafeq_xform* x,
                             const cafeq_quant_cfg* cfg) {
  (void)b; (void)x; (void)cfg;
  if (!a) return 0;
  switch (call_id) {
    case CAFEQ_CALL_RTN_QUANTIZE:
      return align_up(rtn_partials_capacity(a->rows, a->cols) * sizeof(double), 256);
    default:
      return 0;
  }
}

int cafeq_rtn_quantize(const cafeq_mat* W, const cafeq_quant_cfg* cfg, int8_t* codes, float* scales,
                       float* err_sq, void* ws, void* stream) {
  int rc = check_mat(W);
  if (rc) return rc;
  rc = check_cfg(cfg, true);
  if (rc) return rc;
  if (!codes) return CAFEQ_ERR_INVALID_ARG;
  if (!aligned16(codes) || (scales && !aligned16(scales))) return CAFEQ_ERR_BAD_ALIGN;
  const int64_t line = cfg->axis == CAFEQ_AXIS_COL ? W->cols : W->rows;
  const int64_t g = cfg->group == 0 ? line : cfg->group;
  if (line % g != 0) return CAFEQ_ERR_BAD_SHAPE;
  if (err_sq && !ws) return CAFEQ_ERR_WORKSPACE;
  RtnArgs a;
  a.W = W->data; a.dtype = W->dtype; a.rows = W->rows; a.cols = W->cols; a.ld = W->ld;
  a.axis = cfg->axis; a.group = cfg->group; a.grid = make_grid(cfg->bits);
  a.codes = codes; a.scales = scales;
  a.partial = err_sq ? static_cast<double*>(ws) : nullptr;
  a.err_sq = err_sq;
  return launch_rtn(a, static_cast<hipStream_t>(stream));
}

int cafeq_block_inverse(const float* T, int k, int nb, float* Tinv, float* rho_row, float* rho_col,
                        int* status, void* stream) {
  (void)T; (void)k; (void)nb; (void)Tinv; (void)rho_row; (void)rho_col; (void)status; (void)stream;
  return CAFEQ_ERR_UNSUPPORTED;
}

int cafeq_apply_transform(const cafeq_mat* W, const cafeq_xform* x, int axis, int side, float* Z,
                          void* stream) {
  (void)W; (void)x; (void)axis; (void)side; (void)Z; (void)stream;
  return CAFEQ_ERR_UNSUPPORTED;
}

int cafeq_proxy_loss_fwd_bwd(const cafeq_mat* W, const cafeq_xform* x, const cafeq_quant_cfg* cfg,
                             float* losses, float* gradT, int8_t* codes, float* scales, void* ws,
                             void* stream) {
  (void)W; (void)x; (void)cfg; (void)losses; (void)gradT; (void)codes; (void)scales; (void)ws; (void)stream;
  return CAFEQ_ERR_UNSUPPORTED;
}

int cafeq_dual_proxy_loss_fwd_bwd(const cafeq_mat* A, const cafeq_mat* B, const cafeq_xform* x,
                                  const cafeq_quant_cfg* cfg, float lse_t, float* losses, float* gradT,
                                  int8_t* codesU, float* scalesU, int8_t* codesV, float* scalesV,
                                  void* ws, void* stream) {
  (void)A; (void)B; (void)x; (void)cfg; (void)lse_t; (void)losses; (void)gradT; (void)codesU;
  (void)scalesU; (void)codesV; (void)scalesV; (void)ws; (void)stream;
  return CAFEQ_ERR_UNSUPPORTED;
}

int cafeq_adaptive_round_step(const float* U, const float* V, int64_t rowsA, int64_t colsA, int64_t rowsB,
                              int64_t colsB, const cafeq_quant_cfg* cfg, int k, int nb, int rep, int half,
                              int8_t* codesU, float* scalesU, int8_t* codesV, float* scalesV, int* status,
                              void* ws, void* stream) {
  (void)U; (void)V; (void)rowsA; (void)colsA; (void)rowsB; (void)colsB; (void)cfg; (void)k; (void)nb;
  (void)rep; (void)half; (void)codesU; (void)scalesU; (void)codesV; (void)scalesV; (void)status;
  (void)ws; (void)stream;
  return CAFEQ_ERR_UNSUPPORTED;
}

}  // extern "C"
