// Host-side interfaces between the C-ABI layer (cafeq_api.hip) and the kernel files.
#pragma once
#include <algorithm>

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
  double* partial; // workspace for per-workgroup squared-error partials; null = no error output
  float* err_sq;
};
size_t rtn_partials_capacity(int64_t rows, int64_t cols);
int launch_rtn(const RtnArgs& a, hipStream_t st);

}  // namespace cafeq
