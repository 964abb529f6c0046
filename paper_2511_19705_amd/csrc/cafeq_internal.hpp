// Host-side interfaces between the C-ABI layer (cafeq_api.hip) and the kernel files.
#pragma once
#include <algorithm>
#include <atomic>

#include "cafeq_common.hpp"

namespace cafeq {

struct RtnArgs {
  const void* W;
  int dtype;
  int64_t rows, cols, ld;
  int axis;
  int64_t group;  // 0 = whole line
  QGrid grid;
  int8_t* codes;
  float* scales;   // may be null
  float* mins;     // min/max grid only: per-group minimum, may be null
  double* partial; // workspace for per-workgroup squared-error partials; null = no error output
  float* err_sq;
};
size_t rtn_partials_capacity(int64_t rows, int64_t cols);
int launch_rtn_minmax(const RtnArgs& a, int bits, hipStream_t st);
int launch_rtn(const RtnArgs& a, hipStream_t st);


// ---------------------------------------------------------------------------
// fused transform core (xform_core.hpp, instantiated per block size in xform_k*.hip)
// ---------------------------------------------------------------------------
struct CoreParams;
// Launches the core for (K, G, axis); returns CAFEQ_ERR_UNSUPPORTED when that combination
// has no instantiation or its LDS footprint does not fit.
int launch_core(int K, int G, int axis, const CoreParams& p, hipStream_t st);
int launch_core_k32(int G, int axis, const CoreParams& p, hipStream_t st);
int launch_core_k64(int G, int axis, const CoreParams& p, hipStream_t st);
int launch_core_k128(int G, int axis, const CoreParams& p, hipStream_t st);
int launch_core_k256(int G, int axis, const CoreParams& p, hipStream_t st);
// the same on the min/max grid of Eq. (1) (p.asym; gradient-free variants)
int launch_core_asym_k32(int G, int axis, const CoreParams& p, hipStream_t st);
int launch_core_asym_k64(int G, int axis, const CoreParams& p, hipStream_t st);
int launch_core_asym_k128(int G, int axis, const CoreParams& p, hipStream_t st);
int launch_core_asym_k256(int G, int axis, const CoreParams& p, hipStream_t st);
// gradient pass of the two-pass scheme (grad_core.hpp): any block size, p.grp = group length
int launch_grad_pass(int K, int axis, const CoreParams& p, hipStream_t st);
size_t grad_pass_part_floats(int K);
// records of the segments of every group -> one record per group (groups spanning gspan segments of L);
// rec_mm / grec_mm (may be null): the segments' (min, max) pairs and their combination
int launch_combine_records(const float2* rec, int gspan, int L, int64_t nlines, int64_t ngroups, float2* grec,
                           hipStream_t st, const float2* rec_mm = nullptr, float2* grec_mm = nullptr);
// LDS bytes the core needs (0 if the gradient accumulator cannot fit with do_grad)
size_t core_lds_bytes(int K, int G, bool do_grad);
size_t core_lds_bytes_k32(int G, bool do_grad);
size_t core_lds_bytes_k64(int G, bool do_grad);
size_t core_lds_bytes_k128(int G, bool do_grad);
size_t core_lds_bytes_k256(int G, bool do_grad);
int device_cu_count();

// loss_v2.hip: loss pass over prepared weights (128 x 128 blocks, groups up to 128)
// header (||W||^2), per-line factors, the loss pass's tiles, their partial sums, the gradient pass's tiles
struct PreparedLayout { int64_t nlp, nseg, ntiles; size_t off_lscale, off_planes, off_partial, off_gtiles, bytes; };
PreparedLayout prepared_layout(int64_t nlines, int64_t naxis);
int launch_prepare(const cafeq_mat* W, int axis, void* prepared, hipStream_t st);
// gradient pass over prepared weights (blocks of 128; grad_v2.hip): p.prep_gtiles, p.rec, p.grp as launch_grad_pass
size_t prepared_gtiles_bytes(int64_t nlines, int64_t naxis);
int launch_prepare_gtiles(const cafeq_mat* W, int axis, unsigned char* gtiles, hipStream_t st);
int launch_grad_v2(const CoreParams& p, hipStream_t st);
// the same with one workgroup per (matrix, block of 128) and the gradient written in its final form (no partials):
// up to two matrices per launch; the coefficients must be final when it starts (kLossLse: lse_ms = {m*, S})
struct GradOwnerJob {
  const unsigned char* gtiles; const float2* rec; const float* rG; float* out;
  int64_t nlines; int nseg, grp, transpose_out;
};
struct LossArgs;   // loss_reduce.hpp; fold != nullptr: the loss reduction runs inside the launch
int launch_grad_v2_owner(const GradOwnerJob* jobs, int n, int loss_kind, float beta, float lse_t, const double* lse_ms,
                         hipStream_t st, const LossArgs* fold = nullptr);
int launch_loss_v2(int G, int axis, const CoreParams& p, hipStream_t st);
int launch_loss_prepared(int G, int axis, const CoreParams& p, hipStream_t st);   // ... with the caller's timing events
// both members of a pair in one launch (loss_v2.hip), plain and with the caller's timing events
int launch_loss_v2_pair(int G, const CoreParams& pa, const CoreParams& pb, hipStream_t st);
int launch_loss_prepared_pair(int G, const CoreParams& pa, const CoreParams& pb, hipStream_t st);

// aux_kernels.hip
// fscale != null: two float16 planes of the block scaled by a power of two; fscale[block] = the factor back.
// natural: a lane's eight inputs of an MFMA step are consecutive (16c + 8h + 0..7: operands read as prepared
// 16-byte vectors) instead of two runs of four (16c + 8u + 4h + e: operands read as float4 from float32 lines
// and the accumulator registers of the inverse transform).
// texp: a float16 job scales the block's largest magnitude into [2^texp, 2^(texp+1)).
struct SplitRequest { const float* src; uint16_t* dst; int trans, nplanes; float* fscale = nullptr; int natural = 0; int texp = 14; };
int launch_split_planes(const float* src, int K, int nb, int trans, int nplanes, uint16_t* dst, hipStream_t st);
// up to four splits in one launch; hdr (may be null): nslot partial headers reset by the same launch
int launch_split_planes_multi(const SplitRequest* req, int n, int K, int nb, hipStream_t st, float* hdr = nullptr,
                              int64_t nslot = 0);
bool rho_groups_inline(int K, int nb, int G, int rep);
int launch_rho(const float* P, int K, int nb, int by_row, float* rho, hipStream_t st, float* rG = nullptr, int G = 0,
               int rep = 1);   // rG: also the sums over groups of G indices, where rho_groups_inline (see rho_kernel)
int launch_rho_groups(const float* rho, int K, int rep, int G, int64_t ngroups, float* rG, hipStream_t st);
int launch_reduce_grad(const CoreParams& p, int K, int G, bool fused, int nb, int transpose_out,
                       const double* lse_ms, const float* member_ref, float* out, hipStream_t st);
int launch_reduce_grad_pair(const CoreParams& pa, int GA, bool fusedA, const float* refA, float* outA,
                            const CoreParams& pb, int GB, bool fusedB, const float* refB, float* outB, int K,
                            int nb, const double* lse_ms, hipStream_t st);
int launch_build_mmid(const CoreParams& p, int K, int G, int nb, const float* P, int scale_rows, float* Mmid,
                      hipStream_t st);
// gradient reduction + middle factor of the rho path + loss reduction of a single matrix in one launch
int launch_single_tail(const CoreParams& pgrad, const CoreParams& ploss, int K, int G, bool fused, int nb,
                       int transpose_out, float* gradT, const float* P, int scale_rows, float* Mmid, float beta,
                       int nslot, float* losses, double* lse_ms, hipStream_t st);
int launch_reduce_losses(int kind, const float* hdrA, int nslotA, const float* hdrB, int nslotB, float beta,
                         float t, int64_t ngroups, float* losses, double* lse_ms, hipStream_t st);
// Adam step applied by the product's epilogue instead of storing the product: the value alpha op(A) op(B) + beta C is
// taken as the gradient of element [b][i][j] and T, m, v are updated in place (C is only read).  K >= 64.
struct AdamHook { float *T, *m, *v; float lr, beta1, omb1, beta2, omb2, eps, c1, c2; };
// C = alpha op(A) op(B) + beta D per block (D null: C); skip: per-block flags, set = leave the block alone
int launch_bgemm(bool ta, bool tb, const float* A, const float* B, float* C, int K, int nb, float alpha,
                 float beta, hipStream_t st, const AdamHook* adam = nullptr, const float* D = nullptr,
                 const int* skip = nullptr);
int launch_bgemm_chain(const float* P, const float* G, float* x1, float* C, int K, int nb, float alpha, float beta,
                       hipStream_t st, const AdamHook* adam = nullptr);
// adaptive_kernels.hip
int launch_gram_pair(int axis, const float* X, const int8_t* codes, const float* scales, int64_t rows,
                     int64_t cols, int K, int G, int nb, int rep, int64_t chunk, int nchunk, float* partial,
                     hipStream_t st);
int launch_gj_solve(int K, int nb, int nz, const float* partial, double* work, float* Sinv, float* R,
                    float* out, int* status, int status_stride, int status_offset, hipStream_t st);
// inside a learning loop: Tinv holds the previous inverse on entry (Newton warm start, elimination as fallback);
// accurate to about 3e-6 relative
int launch_block_inverse_warm(const float* T, int K, int nb, double* work, float* Tinv, int* status, hipStream_t st);
int launch_block_inverse(const float* T, int K, int nb, double* work, float* Tinv, float* rho_row,
                         float* rho_col, int* status, hipStream_t st);

int launch_pqe(const float* U, const float* V, int64_t rowsA, int64_t colsA, int64_t rowsB, int64_t colsB, int K,
               int GA, int GB, int nb, int rep, const int8_t* codesU, const float* scalesU, const int8_t* codesV,
               const float* scalesV, int64_t chunkA, int nchunkA, int64_t chunkB, int nchunkB, float* partialU,
               float* partialV, double* sums, float* out, hipStream_t st);
int launch_fill(float* p, float value, int64_t n, hipStream_t st);
// blocks smaller than 32 as block-diagonal blocks of 32 (opt_kernels.hip): T32[nb32][32][32] from T[nb][k][k]
// (row-block q of the small transform uses block q / rep); G[nb][k][k] gathered from the diagonal sub-blocks
int launch_embed_blocks(const float* T, int k, int nb, int rep, int nb32, float* T32, hipStream_t st);
int launch_gather_blocks(const float* G32, int k, int nb, int rep, float* G, hipStream_t st);
int launch_expand_status(const int* st32, int m, int nb, int* status, hipStream_t st);
int launch_axpy(float* y, const float* x, float alpha, int64_t n, hipStream_t st);   // y += alpha x
size_t orth_workspace_bytes(int k, int nb);
int launch_div_by_device_scalar(float* g, const float* denom, int64_t n, hipStream_t st);
}  // namespace cafeq
