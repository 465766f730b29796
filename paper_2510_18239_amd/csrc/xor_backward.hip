// Backward pass of one XORA layer with respect to its projected inputs (Appendix H.2), fp32 arithmetic on the
// vector ALUs with the attention matrices recomputed tile by tile (nothing of size N x m is stored).
//
// The layer is symmetric in its two sides (Appendix H.1): with X one side and Y the other,
//   O[Y] = phi(Q[Y] K[X]^T) V[X]   (normaliser n_X, the number of valid rows of X),
//   O[X] = phi(Q[X] K[Y]^T) V[Y]   (normaliser n_Y),                       phi = SiLU(scale .) / n.
// The gradients of side X's own tensors, for its row r and every row c of Y, with G = dL/dO:
//   z1 = scale <Q[Y]_c, K[X]_r>,  p1 = SiLU(z1) / n_X,  e1 = <G[Y]_c, V[X]_r> SiLU'(z1) / n_X
//       dV[X]_r += p1 G[Y]_c,     dK[X]_r += scale e1 Q[Y]_c
//   z2 = scale <Q[X]_r, K[Y]_c>,  e2 = <G[X]_r, V[Y]_c> SiLU'(z2) / n_Y
//       dQ[X]_r += scale e2 K[Y]_c
// (phi' applied element-wise; SiLU'(x) = s (1 + x (1 - s)), s = sigmoid(x)).  One kernel does this for a block of
// 32 rows of X against a range of rows of Y; it runs once with X = history rows (all links as Y, results stored
// directly) and once with X = links (the history rows as Y, cut into chunks whose partial sums a second kernel adds
// in ascending order: deterministic, no atomics).
#include "common.hpp"

namespace lime {
namespace {

constexpr int kOwn = 32;    // rows of X per workgroup
constexpr int kOther = 16;  // rows of Y per step
constexpr int kMaxDh = 64;  // head width the LDS tiles are sized for
constexpr int kColsPerThread = kMaxDh / 8;

struct SideArgs {
  const void *qx, *kx, *vx, *gx;  // [B][rows_x][d]; gx nullable (no upstream gradient for O[X])
  const void *qy, *ky, *vy, *gy;  // [B][rows_y][d]; gy nullable
  void *dq, *dk, *dv;             // [B][rows_x][d], storage type: written when chunks == 1
  float* partial;                 // [B][chunks][3][rows_x][d]: written when chunks > 1
  const int32_t* lens;            // valid history rows per user, nullable = all
  int own_is_history;             // which side the lengths apply to
  int rows_x, rows_y, d, dh, chunks, chunk_rows;  // chunk_rows: rows of Y per chunk, a multiple of kOther
  float scale;
};

__device__ __forceinline__ float silu_f(float x) { return x / (1.f + __expf(-x)); }
__device__ __forceinline__ float silu_derivative_f(float x) {
  const float s = 1.f / (1.f + __expf(-x));
  return s * (1.f + x * (1.f - s));
}

template <typename T>
__global__ __launch_bounds__(256) void xor_backward_side_kernel(SideArgs a) {
  __shared__ float own[4][kOwn][kMaxDh + 1];      // q, k, v, g of the block's rows of X (head slice)
  __shared__ float other[4][kOther][kMaxDh + 1];  // q, k, v, g of the current rows of Y
  __shared__ float p1[kOwn][kOther + 1], e1[kOwn][kOther + 1], e2[kOwn][kOther + 1];
  const int tid = threadIdx.x, dh = a.dh, d = a.d;
  const int blocks_x = (a.rows_x + kOwn - 1) / kOwn;
  const int xb = blockIdx.x % blocks_x, chunk = blockIdx.x / blocks_x, head = blockIdx.y, b = blockIdx.z;
  const int len = a.lens ? min(max(a.lens[b], 0), a.own_is_history ? a.rows_x : a.rows_y) : (a.own_is_history ? a.rows_x : a.rows_y);
  const int valid_x = a.own_is_history ? len : a.rows_x, valid_y = a.own_is_history ? a.rows_y : len;
  const float inv_nx = valid_x > 0 ? 1.f / static_cast<float>(valid_x) : 0.f;
  const float inv_ny = valid_y > 0 ? 1.f / static_cast<float>(valid_y) : 0.f;
  const int r0 = xb * kOwn;
  const int64_t x_base = (static_cast<int64_t>(b) * a.rows_x + r0) * d + head * dh;
  const T* own_src[4] = {static_cast<const T*>(a.qx), static_cast<const T*>(a.kx), static_cast<const T*>(a.vx),
                         static_cast<const T*>(a.gx)};
  const T* other_src[4] = {static_cast<const T*>(a.qy), static_cast<const T*>(a.ky), static_cast<const T*>(a.vy),
                           static_cast<const T*>(a.gy)};
  // rows past the valid ones (padding, or past the end of the tensor) are never read: they count as zeros
  for (int i = tid; i < 4 * kOwn * dh; i += 256) {
    const int w = i / (kOwn * dh), r = (i / dh) % kOwn, t = i % dh;
    own[w][r][t] = (own_src[w] != nullptr && r0 + r < valid_x) ? to_float(own_src[w][x_base + static_cast<int64_t>(r) * d + t]) : 0.f;
  }
  // thread (r, tc) owns columns tc, tc + 8, ... of row r of the three outputs
  const int r = tid / 8, tc = tid % 8;
  float dq[kColsPerThread], dk[kColsPerThread], dv[kColsPerThread];
#pragma unroll
  for (int j = 0; j < kColsPerThread; ++j) dq[j] = dk[j] = dv[j] = 0.f;

  const int c_begin = chunk * a.chunk_rows, c_end = min(c_begin + a.chunk_rows, valid_y);
  for (int c0 = c_begin; c0 < c_end; c0 += kOther) {
    __syncthreads();  // the previous step is done with `other`, p1, e1, e2 (and `own` is complete)
    const int64_t y_base = (static_cast<int64_t>(b) * a.rows_y + c0) * d + head * dh;
    for (int i = tid; i < 4 * kOther * dh; i += 256) {
      const int w = i / (kOther * dh), c = (i / dh) % kOther, t = i % dh;
      other[w][c][t] = (other_src[w] != nullptr && c0 + c < c_end) ? to_float(other_src[w][y_base + static_cast<int64_t>(c) * d + t]) : 0.f;
    }
    __syncthreads();
    // the kOwn x kOther pairs of this step, two per thread
    for (int pair = tid; pair < kOwn * kOther; pair += 256) {
      const int pr = pair / kOther, pc = pair % kOther;
      float z1 = 0.f, w1 = 0.f, z2 = 0.f, w2 = 0.f;
      for (int t = 0; t < dh; ++t) {
        z1 = fmaf(other[0][pc][t], own[1][pr][t], z1);  // <Q[Y]_c, K[X]_r>
        w1 = fmaf(other[3][pc][t], own[2][pr][t], w1);  // <G[Y]_c, V[X]_r>
        z2 = fmaf(own[0][pr][t], other[1][pc][t], z2);  // <Q[X]_r, K[Y]_c>
        w2 = fmaf(own[3][pr][t], other[2][pc][t], w2);  // <G[X]_r, V[Y]_c>
      }
      z1 *= a.scale, z2 *= a.scale;
      const bool live = r0 + pr < valid_x && c0 + pc < c_end;
      p1[pr][pc] = live ? silu_f(z1) * inv_nx : 0.f;
      e1[pr][pc] = live ? w1 * silu_derivative_f(z1) * inv_nx * a.scale : 0.f;
      e2[pr][pc] = live ? w2 * silu_derivative_f(z2) * inv_ny * a.scale : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kColsPerThread; ++j) {
      const int t = tc + 8 * j;
      if (t < dh) {
        for (int c = 0; c < kOther; ++c) {
          dv[j] = fmaf(p1[r][c], other[3][c][t], dv[j]);
          dk[j] = fmaf(e1[r][c], other[0][c][t], dk[j]);
          dq[j] = fmaf(e2[r][c], other[1][c][t], dq[j]);
        }
      }
    }
  }
  if (r0 + r >= a.rows_x) return;
  const int64_t row = static_cast<int64_t>(b) * a.rows_x + r0 + r;
#pragma unroll
  for (int j = 0; j < kColsPerThread; ++j) {
    const int t = tc + 8 * j;
    if (t >= dh) continue;
    const int64_t at = row * d + head * dh + t;
    if (a.chunks == 1) {
      store_as(static_cast<T*>(a.dq) + at, dq[j]);
      store_as(static_cast<T*>(a.dk) + at, dk[j]);
      store_as(static_cast<T*>(a.dv) + at, dv[j]);
    } else {
      const int64_t plane = static_cast<int64_t>(a.rows_x) * d;
      float* dst = a.partial + ((static_cast<int64_t>(b) * a.chunks + chunk) * 3) * plane +
                   static_cast<int64_t>(r0 + r) * d + head * dh + t;
      dst[0] = dq[j], dst[plane] = dk[j], dst[2 * plane] = dv[j];
    }
  }
}

// out[b][which][row][col] = sum over the chunks, in ascending order
template <typename T>
__global__ __launch_bounds__(256) void xor_backward_reduce_kernel(const float* partial, T* dq, T* dk, T* dv, int chunks,
                                                                  int64_t plane) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int which = blockIdx.y, b = blockIdx.z;
  if (i >= plane) return;
  float sum = 0.f;
  for (int c = 0; c < chunks; ++c) sum += partial[((static_cast<int64_t>(b) * chunks + c) * 3 + which) * plane + i];
  T* out = which == 0 ? dq : (which == 1 ? dk : dv);
  store_as(out + static_cast<int64_t>(b) * plane + i, sum);
}

int chunks_for_links(int B, int N, int m, int h) {
  // enough workgroups for two per compute unit, but no chunk shorter than one step
  const int64_t per_chunk = static_cast<int64_t>((m + kOwn - 1) / kOwn) * h * B;
  int64_t chunks = (2 * static_cast<int64_t>(compute_units()) + per_chunk - 1) / per_chunk;
  const int64_t steps = (N + kOther - 1) / kOther;
  if (chunks > steps) chunks = steps;
  if (chunks < 1) chunks = 1;
  return static_cast<int>(chunks);
}

template <typename T>
hipError_t xor_backward_typed(const XorBackward& g, void* workspace, hipStream_t s) {
  SideArgs a{};
  a.lens = g.lens, a.d = g.d, a.dh = g.d / g.h, a.scale = g.scale;
  // history side: every block of 32 history rows against all links
  a.qx = g.QS, a.kx = g.KS, a.vx = g.VS, a.gx = g.dOS;
  a.qy = g.QT, a.ky = g.KT, a.vy = g.VT, a.gy = g.dOT;
  a.dq = g.dQS, a.dk = g.dKS, a.dv = g.dVS, a.partial = nullptr;
  a.own_is_history = 1, a.rows_x = g.N, a.rows_y = g.m, a.chunks = 1;
  a.chunk_rows = (g.m + kOther - 1) / kOther * kOther;
  hipLaunchKernelGGL(xor_backward_side_kernel<T>, dim3((g.N + kOwn - 1) / kOwn, g.h, g.B), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // link side: every block of 32 links against the history rows, in chunks
  const int chunks = chunks_for_links(g.B, g.N, g.m, g.h);
  a.qx = g.QT, a.kx = g.KT, a.vx = g.VT, a.gx = g.dOT;
  a.qy = g.QS, a.ky = g.KS, a.vy = g.VS, a.gy = g.dOS;
  a.dq = g.dQT, a.dk = g.dKT, a.dv = g.dVT, a.partial = static_cast<float*>(workspace);
  a.own_is_history = 0, a.rows_x = g.m, a.rows_y = g.N, a.chunks = chunks;
  const int steps = (g.N + kOther - 1) / kOther;
  a.chunk_rows = (steps + chunks - 1) / chunks * kOther;
  const int blocks_x = (g.m + kOwn - 1) / kOwn;
  hipLaunchKernelGGL(xor_backward_side_kernel<T>, dim3(blocks_x * chunks, g.h, g.B), dim3(256), 0, s, a);
  e = hipGetLastError();
  if (e != hipSuccess || chunks == 1) return e;
  const int64_t plane = static_cast<int64_t>(g.m) * g.d;
  hipLaunchKernelGGL(xor_backward_reduce_kernel<T>, dim3(static_cast<unsigned>((plane + 255) / 256), 3, g.B), dim3(256), 0, s,
                     static_cast<const float*>(workspace), static_cast<T*>(g.dQT), static_cast<T*>(g.dKT),
                     static_cast<T*>(g.dVT), chunks, plane);
  return hipGetLastError();
}

}  // namespace

bool xor_backward_supported(int d, int h) { return h > 0 && d % h == 0 && d / h <= kMaxDh; }

size_t xor_backward_workspace(int B, int N, int m, int d, int h) {
  const int chunks = chunks_for_links(B, N, m, h);
  return chunks == 1 ? 256 : align_up(static_cast<size_t>(B) * chunks * 3 * m * d * sizeof(float));
}

hipError_t xor_backward(const XorBackward& g, void* workspace, hipStream_t s) {
  return g.dtype == 0 ? xor_backward_typed<float>(g, workspace, s) : xor_backward_typed<bf16_t>(g, workspace, s);
}

}  // namespace lime
