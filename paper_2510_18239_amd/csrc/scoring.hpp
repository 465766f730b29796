// Launcher interface of the scoring pipeline around the attention stages (scoring.hip).
#pragma once

#include "mfma.hpp"

namespace lime {

// Y = LayerNorm(X; gamma, beta, eps) row by row over d features (gamma, beta in the storage type, nullable = 1 / 0).
// With lens, row r belongs to user r / rows_per_user and is skipped (neither read nor written) when its index within
// the user is at or past lens[user].
hipError_t layer_norm_rows(const void* X, const void* gamma, const void* beta, float eps, void* Y, int64_t rows, int d,
                           const int32_t* lens, int rows_per_user, int dtype, hipStream_t s);

// Y[r] = act([X1[r % x1_rows] | X2[r / x2_rows_per]] W + b), fp32 arithmetic; storage types 0 = fp32, 1 = bf16.
struct Dense {
  const void* X1;
  int64_t x1_rows;   // 0 = rows
  const void* X2;    // nullable
  int x2_rows_per;
  const void *W, *b; // [d1 + d2][dout], [dout] (nullable)
  void* Y;
  int64_t rows;
  int d1, d2, dout;
  bool relu;
  int x_dtype, w_dtype, y_dtype;
};
hipError_t dense_rows(const Dense& q, hipStream_t s);

// The interaction network on the matrix cores (bf16): n_maps affine maps, widths[i] outputs each, the last to one logit.
bool interaction_mlp_on_matrix_cores(int d, int n_maps, const int32_t* widths);
size_t interaction_mlp_image_bytes(int d, int n_maps, const int32_t* widths);
hipError_t interaction_mlp_mfma(const void* O, int64_t rows, int d, int n_maps, const int32_t* widths, const void* const* W,
                                const void* const* b, float* scores, void* images, hipStream_t s);

}  // namespace lime
