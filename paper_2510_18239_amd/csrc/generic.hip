// General kernels: fp32 arithmetic on the vector ALUs, any shape with d/h <= 256.
// They serve the fp32 storage type and every bf16 shape the matrix-core kernels do
// not cover.  Each step is the plain definition (Eq. 1): a projection X~ = X W and an
// attention (phi(scale * Q~ K~^T) restricted to the valid keys) V~.
#include "common.hpp"

namespace lime {
namespace {

// ----------------------------------------------------------------------------- projection
constexpr int PT = 64;  // output tile edge
constexpr int PK = 16;  // k-slice

template <typename T>
__global__ __launch_bounds__(256) void project_kernel(const T* __restrict__ X, const T* __restrict__ W,
                                                      float* __restrict__ Y, int64_t rows, int d) {
  __shared__ float Xs[PK][PT + 1];
  __shared__ float Ws[PK][PT + 1];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * PT;
  const int c0 = blockIdx.y * PT;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < d; k0 += PK) {
    for (int idx = threadIdx.x; idx < PT * PK; idx += 256) {
      const int r = idx / PK, k = idx % PK;  // X tile: consecutive threads walk k
      const int64_t row = r0 + r;
      Xs[k][r] = (row < rows && k0 + k < d) ? to_float(X[row * d + k0 + k]) : 0.f;
      const int kk = idx / PT, c = idx % PT;  // W tile: consecutive threads walk c
      Ws[kk][c] = (k0 + kk < d && c0 + c < d) ? to_float(W[static_cast<int64_t>(k0 + kk) * d + c0 + c]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < PK; ++k) {
      float xv[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) xv[i] = Xs[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) wv[j] = Ws[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(xv[i], wv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = r0 + ty * 4 + i;
    if (row >= rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = c0 + tx * 4 + j;
      if (c < d) Y[row * d + c] = acc[i][j];
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void upcast_kernel(const T* __restrict__ X, float* __restrict__ Y, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) Y[i] = to_float(X[i]);
}

// ----------------------------------------------------------------------------- attention
constexpr int QT = 16;    // query rows per block
constexpr int KT = 64;    // keys per step
constexpr int MAXOUT = 16;  // outputs per thread: QT * (d/h) / 256 <= 16 for d/h <= 256

struct AttnDev {
  const float *Q, *K, *V;
  int64_t qs, ks, vs;
  void* O;
  const int32_t *q_lens, *k_lens;
  int q_rows, n_keys, d, dh;
  float scale;
};

template <typename OutT, int PHI>
__global__ __launch_bounds__(256) void attention_kernel(AttnDev a) {
  extern __shared__ float smem[];
  float* Qs = smem;                  // [QT][dh], already multiplied by scale
  float* S = Qs + QT * a.dh;         // [QT][KT] logits, then weights
  float* row_max = S + QT * KT;      // [QT]
  float* row_sum = row_max + QT;     // [QT]
  float* row_alpha = row_sum + QT;   // [QT]

  const int tid = threadIdx.x;
  const int b = blockIdx.z, head = blockIdx.y, q0 = blockIdx.x * QT;
  const int dh = a.dh, d = a.d;
  const int qlen = a.q_lens ? min(a.q_lens[b], a.q_rows) : a.q_rows;
  const int klen = a.k_lens ? min(a.k_lens[b], a.n_keys) : a.n_keys;
  const float* Qb = a.Q + b * a.qs + head * dh;
  const float* Kb = a.K + b * a.ks + head * dh;
  const float* Vb = a.V + b * a.vs + head * dh;

  for (int idx = tid; idx < QT * dh; idx += 256) {
    const int i = idx / dh, t = idx % dh, row = q0 + i;
    Qs[idx] = row < qlen ? Qb[static_cast<int64_t>(row) * d + t] * a.scale : 0.f;
  }
  if (tid < QT) {
    row_max[tid] = -INFINITY;
    row_sum[tid] = 0.f;
  }
  float acc[MAXOUT];
#pragma unroll
  for (int u = 0; u < MAXOUT; ++u) acc[u] = 0.f;
  __syncthreads();

  for (int k0 = 0; k0 < klen; k0 += KT) {
    const int kn = min(KT, klen - k0);
    // logits of this key block
    for (int idx = tid; idx < QT * KT; idx += 256) {
      const int i = idx / KT, j = idx % KT;
      float s = -INFINITY;
      if (j < kn) {
        const float* kr = Kb + static_cast<int64_t>(k0 + j) * d;
        const float* qr = Qs + i * dh;
        s = 0.f;
        for (int t = 0; t < dh; ++t) s = fmaf(qr[t], kr[t], s);
      }
      S[idx] = s;
    }
    __syncthreads();
    // phi: 16 lanes share one query row
    {
      const int i = tid / 16, l = tid % 16;
      float v[KT / 16];
#pragma unroll
      for (int u = 0; u < KT / 16; ++u) v[u] = S[i * KT + l + 16 * u];
      if (PHI == kPhiSoftmax) {
        float cmax = v[0];
#pragma unroll
        for (int u = 1; u < KT / 16; ++u) cmax = fmaxf(cmax, v[u]);
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, off, 16));
        const float old_max = row_max[i];
        const float new_max = fmaxf(old_max, cmax);  // finite: the block holds at least one valid key
        float csum = 0.f;
#pragma unroll
        for (int u = 0; u < KT / 16; ++u) {
          v[u] = expf(v[u] - new_max);  // masked logits are -inf -> 0
          csum += v[u];
        }
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) csum += __shfl_xor(csum, off, 16);
        const float alpha = expf(old_max - new_max);  // old_max = -inf on the first block -> 0
        if (l == 0) {
          row_max[i] = new_max;
          row_sum[i] = row_sum[i] * alpha + csum;
          row_alpha[i] = alpha;
        }
      } else {
#pragma unroll
        for (int u = 0; u < KT / 16; ++u) {
          const bool valid = l + 16 * u < kn;
          v[u] = valid ? v[u] / (1.f + expf(-v[u])) : 0.f;
        }
        if (l == 0) row_alpha[i] = 1.f;
      }
#pragma unroll
      for (int u = 0; u < KT / 16; ++u) S[i * KT + l + 16 * u] = v[u];
    }
    __syncthreads();
    // weighted sum of the value rows
#pragma unroll
    for (int u = 0; u < MAXOUT; ++u) {
      const int o = tid + u * 256;
      if (o < QT * dh) {
        const int i = o / dh, t = o % dh;
        float x = acc[u] * row_alpha[i];
        const float* w = S + i * KT;
        const float* vr = Vb + static_cast<int64_t>(k0) * d + t;
        for (int j = 0; j < kn; ++j) x = fmaf(w[j], vr[static_cast<int64_t>(j) * d], x);
        acc[u] = x;
      }
    }
    __syncthreads();
  }

  OutT* Ob = static_cast<OutT*>(a.O) + (static_cast<int64_t>(b) * a.q_rows) * d + head * dh;
#pragma unroll
  for (int u = 0; u < MAXOUT; ++u) {
    const int o = tid + u * 256;
    if (o < QT * dh) {
      const int i = o / dh, t = o % dh, row = q0 + i;
      if (row >= a.q_rows) continue;
      float x = 0.f;
      if (row < qlen && klen > 0) x = PHI == kPhiSoftmax ? acc[u] / row_sum[i] : acc[u] / static_cast<float>(klen);
      store_as(Ob + static_cast<int64_t>(row) * d + t, x);
    }
  }
}

template <typename OutT, int PHI>
hipError_t launch_attention(const AttnDev& dev, int B, int h, hipStream_t s) {
  const size_t smem = (static_cast<size_t>(QT) * dev.dh + QT * KT + 3 * QT) * sizeof(float);
  dim3 grid((dev.q_rows + QT - 1) / QT, h, B);
  hipLaunchKernelGGL((attention_kernel<OutT, PHI>), grid, dim3(256), smem, s, dev);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- QK cache (Section 3.3)
// One wave per (user, candidate, head): weights = softmax over the m links of the scaled logits.
template <typename OutT>
__global__ __launch_bounds__(256) void qk_weights_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                                                         OutT* __restrict__ W, int64_t rows, int d, int h, int m,
                                                         float scale) {
  const int lane = threadIdx.x & 63;
  const int64_t item = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);  // (row, head)
  if (item >= rows * h) return;
  const int64_t row = item / h;
  const int head = static_cast<int>(item % h), dh = d / h;
  const float* q = Q + row * d + head * dh;
  float mx = -INFINITY;
  for (int i = lane; i < m; i += 64) {
    const float* k = K + static_cast<int64_t>(i) * d + head * dh;
    float s = 0.f;
    for (int t = 0; t < dh; ++t) s = fmaf(q[t], k[t], s);
    mx = fmaxf(mx, s * scale);
  }
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  float sum = 0.f;
  for (int i = lane; i < m; i += 64) {
    const float* k = K + static_cast<int64_t>(i) * d + head * dh;
    float s = 0.f;
    for (int t = 0; t < dh; ++t) s = fmaf(q[t], k[t], s);
    sum += expf(s * scale - mx);
  }
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  for (int i = lane; i < m; i += 64) {
    const float* k = K + static_cast<int64_t>(i) * d + head * dh;
    float s = 0.f;
    for (int t = 0; t < dh; ++t) s = fmaf(q[t], k[t], s);
    store_as(W + (row * h + head) * m + i, expf(s * scale - mx) / sum);
  }
}

// One thread per output element: O[b][c][col] = sum_i W[b][c][head(col)][i] * V[b][i][col]; with ids, the
// weight row is row ids[b][c] of a table of n_items rows, and an id outside the table gives zero.
template <typename T>
__global__ __launch_bounds__(256) void cached_sum_kernel(const T* __restrict__ W, const int32_t* __restrict__ ids,
                                                         int n_items, const float* __restrict__ V, T* __restrict__ O,
                                                         int64_t total, int C, int d, int h, int m) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= total) return;
  const int col = static_cast<int>(idx % d);
  const int64_t row = idx / d, b = row / C;
  const int head = col / (d / h);
  int64_t wrow = row;
  if (ids != nullptr) {
    const int id = ids[row];
    if (static_cast<unsigned>(id) >= static_cast<unsigned>(n_items)) {
      store_as(O + idx, 0.f);
      return;
    }
    wrow = id;
  }
  const T* w = W + (wrow * h + head) * m;
  const float* v = V + b * m * d + col;
  float acc = 0.f;
  for (int i = 0; i < m; ++i) acc = fmaf(to_float(w[i]), v[static_cast<int64_t>(i) * d], acc);
  store_as(O + idx, acc);
}

}  // namespace

hipError_t generic_qk_weights(const float* Q, const float* K, void* W, int64_t rows, int d, int h, int m, float scale,
                              int dtype, hipStream_t s) {
  const int64_t items = rows * h;
  dim3 grid(static_cast<unsigned>((items + 3) / 4));
  if (dtype == 0)
    hipLaunchKernelGGL(qk_weights_kernel<float>, grid, dim3(256), 0, s, Q, K, static_cast<float*>(W), rows, d, h, m, scale);
  else
    hipLaunchKernelGGL(qk_weights_kernel<bf16_t>, grid, dim3(256), 0, s, Q, K, static_cast<bf16_t*>(W), rows, d, h, m, scale);
  return hipGetLastError();
}

hipError_t generic_cached_sum(const void* W, const int32_t* ids, int n_items, const float* V, void* O, int B, int C,
                              int d, int h, int m, int dtype, hipStream_t s) {
  const int64_t total = static_cast<int64_t>(B) * C * d;
  dim3 grid(static_cast<unsigned>((total + 255) / 256));
  if (dtype == 0)
    hipLaunchKernelGGL(cached_sum_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(W), ids, n_items, V,
                       static_cast<float*>(O), total, C, d, h, m);
  else
    hipLaunchKernelGGL(cached_sum_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t*>(W), ids, n_items, V,
                       static_cast<bf16_t*>(O), total, C, d, h, m);
  return hipGetLastError();
}

hipError_t generic_project(const void* X, const void* W, float* Y, int64_t rows, int d, int dtype, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (W == nullptr) {
    const int64_t n = rows * d;
    dim3 grid(static_cast<unsigned>((n + 255) / 256));
    if (dtype == 0)
      hipLaunchKernelGGL(upcast_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(X), Y, n);
    else
      hipLaunchKernelGGL(upcast_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t*>(X), Y, n);
    return hipGetLastError();
  }
  dim3 grid(static_cast<unsigned>((rows + PT - 1) / PT), (d + PT - 1) / PT);
  if (dtype == 0)
    hipLaunchKernelGGL(project_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(X),
                       static_cast<const float*>(W), Y, rows, d);
  else
    hipLaunchKernelGGL(project_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t*>(X),
                       static_cast<const bf16_t*>(W), Y, rows, d);
  return hipGetLastError();
}

namespace {

// Z = A * SiLU(P), P = X Wu in fp32 (one block of rows for all users when p_user_stride == 0)
template <typename T>
__global__ __launch_bounds__(256) void gate_kernel(const float* __restrict__ P, int64_t p_user_stride, const T* __restrict__ A,
                                                   const int32_t* __restrict__ lens, T* __restrict__ Z, int rows, int d,
                                                   int64_t total) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t per_user = static_cast<int64_t>(rows) * d;
  const int b = static_cast<int>(i / per_user);
  const int64_t rem = i - b * per_user;
  const int row = static_cast<int>(rem / d);
  const bool valid = row < (lens ? min(lens[b], rows) : rows);
  const float p = P[b * p_user_stride + rem];
  store_as(Z + i, valid ? to_float(A[i]) * p / (1.f + expf(-p)) : 0.f);
}

// Y = X + P, P = Z Wo in fp32; the running sum of P over the layers
template <typename T>
__global__ __launch_bounds__(256) void residual_kernel(const float* __restrict__ P, const T* __restrict__ X, int64_t x_user_stride,
                                                       const int32_t* __restrict__ lens, T* __restrict__ Y,
                                                       const float* __restrict__ sum_in, float* __restrict__ sum_out,
                                                       T* __restrict__ sum_rounded, int rows, int d, int64_t total) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t per_user = static_cast<int64_t>(rows) * d;
  const int b = static_cast<int>(i / per_user);
  const int64_t rem = i - b * per_user;
  const int row = static_cast<int>(rem / d);
  const bool valid = row < (lens ? min(lens[b], rows) : rows);
  const float p = P[i];
  if (Y != nullptr) store_as(Y + i, valid ? to_float(X[b * x_user_stride + rem]) + p : 0.f);
  if (sum_out != nullptr || sum_rounded != nullptr) {
    const float t = (sum_in != nullptr ? sum_in[i] : 0.f) + p;
    if (sum_out != nullptr) sum_out[i] = t;
    if (sum_rounded != nullptr) store_as(sum_rounded + i, t);
  }
}

template <typename T>
hipError_t gated_block_typed(const GenericGatedBlock& g, hipStream_t s) {
  const int64_t total = static_cast<int64_t>(g.B) * g.rows * g.d;
  const dim3 grid(static_cast<unsigned>((total + 255) / 256));
  const bool shared = g.x_user_stride == 0;
  hipError_t e = generic_project(g.X, g.Wu, g.P, shared ? g.rows : static_cast<int64_t>(g.B) * g.rows, g.d, g.dtype, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(gate_kernel<T>, grid, dim3(256), 0, s, g.P, shared ? int64_t{0} : static_cast<int64_t>(g.rows) * g.d,
                     static_cast<const T*>(g.A), g.lens, static_cast<T*>(g.Z), g.rows, g.d, total);
  e = generic_project(g.Z, g.Wo, g.P, static_cast<int64_t>(g.B) * g.rows, g.d, g.dtype, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(residual_kernel<T>, grid, dim3(256), 0, s, g.P, static_cast<const T*>(g.X), g.x_user_stride, g.lens,
                     static_cast<T*>(g.Y), g.sum_in, g.sum_out, static_cast<T*>(g.sum_rounded), g.rows, g.d, total);
  return hipGetLastError();
}

}  // namespace

hipError_t generic_gated_block(const GenericGatedBlock& g, hipStream_t s) {
  if (g.B <= 0 || g.rows <= 0) return hipSuccess;
  return g.dtype == 0 ? gated_block_typed<float>(g, s) : gated_block_typed<bf16_t>(g, s);
}

hipError_t generic_attention(const GenericAttention& a, hipStream_t s) {
  if (a.B <= 0 || a.q_rows <= 0) return hipSuccess;
  AttnDev dev{a.Q, a.K, a.V, a.q_user_stride, a.k_user_stride, a.v_user_stride, a.O, a.q_lens, a.k_lens,
              a.q_rows, a.n_keys, a.d, a.d / a.h, a.scale};
  if (a.dtype == 0)
    return a.phi == kPhiSoftmax ? launch_attention<float, kPhiSoftmax>(dev, a.B, a.h, s)
                                : launch_attention<float, kPhiSilu>(dev, a.B, a.h, s);
  return a.phi == kPhiSoftmax ? launch_attention<bf16_t, kPhiSoftmax>(dev, a.B, a.h, s)
                              : launch_attention<bf16_t, kPhiSilu>(dev, a.B, a.h, s);
}

}  // namespace lime
