// Shared device helpers and the internal launcher interface of the LIME HIP library.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace lime {

// ----------------------------------------------------------------------------- storage types
struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(static_cast<uint32_t>(x.bits) << 16); }

// fp32 -> bf16, round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

__device__ __forceinline__ void store_as(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_as(bf16_t* p, float v) { p->bits = f32_to_bf16_bits(v); }

constexpr int kPhiSoftmax = 0;
constexpr int kPhiSilu = 1;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Compute units of the current device (256 when the query fails): what the launchers size their grids by.
int compute_units();
// Sets the calling thread's error text (what lime_last_error returns) and hands the status back.
int32_t set_error(int32_t status, const char* text);

// ----------------------------------------------------------------------------- per-kernel timing (profile.hip)
enum ProfiledKernel { kKernelQueriesOverLinks = 0, kKernelLinksOverHistory = 1, kKernelTargetAttention = 2,
                      kKernelProjection = 3, kKernelCachedCandidates = 4, kKernelProbeCopy = 5, kKernelProbeMfma = 6 };
// When profiling is on: a fresh pair of events for one launch of `kernel`, remembered for lime_profile_collect.
bool profile_events(int kernel, hipEvent_t* start, hipEvent_t* stop);
// Launches a main kernel; with profiling on, the launch carries a start and a stop event of its own, which the
// runtime fills from the dispatch's begin and end time stamps (the kernel's duration as a tracer sees it, without
// the gaps an event recorded before or after the launch would include).
template <typename... KA, typename... A>
inline void launch_timed(int kernel_id, void (*kernel)(KA...), dim3 grid, dim3 block, size_t lds, hipStream_t s, A... args) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (profile_events(kernel_id, &e0, &e1))
    hipExtLaunchKernelGGL(kernel, grid, block, static_cast<uint32_t>(lds), s, e0, e1, 0, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
}

// ----------------------------------------------------------------------------- general kernels (generic.hip)
// Y[rows][d] (fp32) = X[rows][d] * W[d][d]; W == nullptr copies X (identity projection).
hipError_t generic_project(const void* X, const void* W, float* Y, int64_t rows, int d, int dtype, hipStream_t s);

struct GenericAttention {
  const float* Q;      // [.][q_rows][d], user b at Q + b * q_user_stride
  const float* K;      // [.][n_keys][d]
  const float* V;      // [.][n_keys][d]
  int64_t q_user_stride, k_user_stride, v_user_stride;  // in elements; 0 = shared by all users
  void* O;             // [B][q_rows][d] in `dtype`
  const int32_t* q_lens;  // nullable; query rows >= q_lens[b] are written as zeros
  const int32_t* k_lens;  // nullable; keys >= k_lens[b] are masked
  int B, q_rows, n_keys, d, h;
  float scale;
  int phi;    // kPhiSoftmax: softmax over valid keys; kPhiSilu: SiLU(logit) / (number of valid keys)
  int dtype;  // of O
};
hipError_t generic_attention(const GenericAttention& a, hipStream_t s);

// QK cache (Section 3.3): W[rows][h][m] = softmax over m of scale * <Q[row]_head, K[i]_head> (Q, K projected, fp32);
// and the online weighted sum O[b][c][col] = sum_i W[b][c][head(col)][i] * V[b][i][col] (V projected, fp32);
// with ids (nullable) the weight row of (b, c) is row ids[b][c] of a table of n_items rows.
hipError_t generic_qk_weights(const float* Q, const float* K, void* W, int64_t rows, int d, int h, int m, float scale,
                              int dtype, hipStream_t s);
hipError_t generic_cached_sum(const void* W, const int32_t* ids, int n_items, const float* V, void* O, int B, int C,
                              int d, int h, int m, int dtype, hipStream_t s);

// The gated block of an XOR layer (Eq. 8) for any shape and storage type, as two projections with an element-wise
// step after each: Z = A * SiLU(X Wu); Y = X + Z Wo (rows >= lens[b] are zeros); the running sum of the layers'
// outputs as in the matrix-core version.  P (fp32) and Z (storage type) are scratch of B * rows * d elements.
struct GenericGatedBlock {
  const void* X;          // [.][rows][d]
  int64_t x_user_stride;  // elements between users; 0 = one block for all users
  const int32_t* lens;    // nullable
  const void *Wu, *Wo;    // [d][d]
  const void* A;          // [B][rows][d]
  void* Y;                // [B][rows][d], nullable
  const float* sum_in;    // nullable = zero
  float* sum_out;         // nullable
  void* sum_rounded;      // storage type, nullable
  float* P;
  void* Z;
  int B, rows, d, dtype;
};
hipError_t generic_gated_block(const GenericGatedBlock& g, hipStream_t s);

// Gradients of one XORA layer with respect to its projected inputs (Appendix H.2): matrix cores for bf16 storage with
// d/h = 32 or 64, fp32 arithmetic on the vector ALUs otherwise.
struct XorBackward {
  const void *QS, *KS, *VS;     // [B][N][d] projected history rows
  const void *QT, *KT, *VT;     // [B][m][d] projected links, per user
  const void* dOT;              // [B][m][d]
  const void* dOS;              // [B][N][d], nullable: O[S] has no consumer
  const int32_t* lens;          // nullable
  void *dQS, *dKS, *dVS;        // [B][N][d]
  void *dQT, *dKT, *dVT;        // [B][m][d]
  int B, N, m, d, h, dtype;     // dtype: 0 = fp32, 1 = bf16 storage
  float scale;
};
bool xor_backward_supported(int d, int h);  // d/h <= 64
size_t xor_backward_workspace(int B, int N, int m, int d, int h);
hipError_t xor_backward(const XorBackward& g, void* workspace, hipStream_t s);

}  // namespace lime
