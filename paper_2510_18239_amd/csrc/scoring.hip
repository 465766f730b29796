// The scoring pipeline around the two attention stages: layer normalisation of the rows that enter an MHA
// (Appendix C, "Model Design"), the link contextualisation MLP (Section 3.1 Eq. 2) and the interaction network that
// turns a LIME embedding into a score (Section 3.3; widths from the hyper-parameter table of Appendix C).
//
//  * layer_norm_rows: one pass, a row per group of d/8 lanes (16-byte loads and stores), statistics in fp32 from
//    registers (mean first, then the centred second moment).
//  * dense_rows: Y = act(X W + b) in fp32 arithmetic on the vector ALUs for any shape; X may be the concatenation of a
//    row-varying part and a per-user part (Eq. 2's L (+) E^C).  Serves Eq. 2 (a few hundred rows) and, for shapes and
//    storage types the matrix-core kernel does not cover, the interaction network.
//  * interaction_mlp_kernel: the whole interaction network for 32 rows per wavefront on the matrix cores.  The
//    row's embedding is the B operand of the first layer; every layer computes Y^T = W^T X^T, so its accumulators,
//    after bias and ReLU, are as they stand the B operand of the next layer (chained k order, see mfma.hpp) and the
//    hidden activations never leave registers; the last affine map to one logit is a dot product over the lane's
//    registers plus one exchange with lane ^ 32.
#include <type_traits>

#include "scoring.hpp"

namespace lime {
namespace {

// ----------------------------------------------------------------------------- layer normalisation
struct LnArgs {
  const void* X;
  void* Y;
  const void *gamma, *beta;  // [d] in the storage type, nullable
  const int32_t* lens;       // nullable: rows r >= lens[r / rows_per_user] are skipped
  int64_t rows;
  int rows_per_user, d;
  float eps;
};

// bf16, d = 8 G with G a power of two up to 64: G lanes per row, one 16-byte piece each.
template <int G>
__global__ __launch_bounds__(256) void layer_norm_bf16_kernel(LnArgs a) {
  constexpr int D = 8 * G;
  const int sub = threadIdx.x % G;
  const int64_t row = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) / G;
  const bool live = row < a.rows && (a.lens == nullptr || static_cast<int>(row % a.rows_per_user) < a.lens[row / a.rows_per_user]);
  bf16x8 v;
#pragma unroll
  for (int t = 0; t < 8; ++t) v[t] = static_cast<__bf16>(0.f);
  if (live) v = *reinterpret_cast<const bf16x8*>(static_cast<const bf16_t*>(a.X) + row * D + 8 * sub);
  float x[8], s = 0.f;
#pragma unroll
  for (int t = 0; t < 8; ++t) x[t] = static_cast<float>(v[t]), s += x[t];
#pragma unroll
  for (int o = 1; o < G; o *= 2) s += __shfl_xor(s, o, 64);
  const float mean = s * (1.f / D);
  float q = 0.f;
#pragma unroll
  for (int t = 0; t < 8; ++t) x[t] -= mean, q = fmaf(x[t], x[t], q);
#pragma unroll
  for (int o = 1; o < G; o *= 2) q += __shfl_xor(q, o, 64);
  const float inv = 1.f / sqrtf(q * (1.f / D) + a.eps);
  bf16x8 y, gv, bv;
#pragma unroll
  for (int t = 0; t < 8; ++t) gv[t] = static_cast<__bf16>(1.f), bv[t] = static_cast<__bf16>(0.f);
  if (a.gamma != nullptr) gv = *reinterpret_cast<const bf16x8*>(static_cast<const bf16_t*>(a.gamma) + 8 * sub);
  if (a.beta != nullptr) bv = *reinterpret_cast<const bf16x8*>(static_cast<const bf16_t*>(a.beta) + 8 * sub);
#pragma unroll
  for (int t = 0; t < 8; ++t) y[t] = static_cast<__bf16>(fmaf(x[t] * inv, static_cast<float>(gv[t]), static_cast<float>(bv[t])));
  if (live) *reinterpret_cast<bf16x8*>(static_cast<bf16_t*>(a.Y) + row * D + 8 * sub) = y;
}

// any width and storage type: one wavefront per row
template <typename T>
__global__ __launch_bounds__(256) void layer_norm_kernel(LnArgs a) {
  const int lane = threadIdx.x % 64;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + threadIdx.x / 64;
  if (row >= a.rows) return;  // uniform over the wave
  if (a.lens != nullptr && static_cast<int>(row % a.rows_per_user) >= a.lens[row / a.rows_per_user]) return;
  const T* x = static_cast<const T*>(a.X) + row * a.d;
  T* y = static_cast<T*>(a.Y) + row * a.d;
  float s = 0.f;
  for (int k = lane; k < a.d; k += 64) s += to_float(x[k]);
#pragma unroll
  for (int o = 1; o < 64; o *= 2) s += __shfl_xor(s, o, 64);
  const float mean = s / static_cast<float>(a.d);
  float q = 0.f;
  for (int k = lane; k < a.d; k += 64) {
    const float c = to_float(x[k]) - mean;
    q = fmaf(c, c, q);
  }
#pragma unroll
  for (int o = 1; o < 64; o *= 2) q += __shfl_xor(q, o, 64);
  const float inv = 1.f / sqrtf(q / static_cast<float>(a.d) + a.eps);
  for (int k = lane; k < a.d; k += 64) {
    float r = (to_float(x[k]) - mean) * inv;
    if (a.gamma != nullptr) r *= to_float(static_cast<const T*>(a.gamma)[k]);
    if (a.beta != nullptr) r += to_float(static_cast<const T*>(a.beta)[k]);
    store_as(y + k, r);
  }
}

// ----------------------------------------------------------------------------- dense layers, fp32 arithmetic
struct DenseArgs {
  const void* X1;     // [x1_rows][d1]: row r of the product reads row r % x1_rows
  const void* X2;     // nullable: [.][d2], row r reads row r / x2_rows_per: the per-user part of a concatenated input
  const void* W;      // [d1 + d2][dout]
  const void* b;      // [dout], nullable
  void* Y;            // [rows][dout]
  int64_t rows, x1_rows;
  int x2_rows_per, d1, d2, dout, relu;
};

constexpr int kDenseRows = 16, kDenseCols = 64, kDenseK = 16;

// TX: type of X1 / X2; TW: type of W and b; TY: type of Y.
template <typename TX, typename TW, typename TY>
__global__ __launch_bounds__(256) void dense_rows_kernel(DenseArgs a) {
  __shared__ float Xs[kDenseRows][kDenseK + 1];
  __shared__ float Ws[kDenseK][kDenseCols];
  const int tid = threadIdx.x, col = tid % kDenseCols, rg = tid / kDenseCols;  // 4 row groups of 4 rows
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * kDenseRows;
  const int c0 = blockIdx.y * kDenseCols, din = a.d1 + a.d2;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < din; k0 += kDenseK) {
    {
      const int r = tid / kDenseK, k = k0 + tid % kDenseK;
      const int64_t row = r0 + r;
      float v = 0.f;
      if (row < a.rows && k < din) {
        if (k < a.d1)
          v = to_float(static_cast<const TX*>(a.X1)[(row % a.x1_rows) * a.d1 + k]);
        else
          v = to_float(static_cast<const TX*>(a.X2)[(row / a.x2_rows_per) * a.d2 + (k - a.d1)]);
      }
      Xs[r][tid % kDenseK] = v;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + 256 * i, kk = idx / kDenseCols, c = idx % kDenseCols;
      Ws[kk][c] = (k0 + kk < din && c0 + c < a.dout)
                      ? to_float(static_cast<const TW*>(a.W)[static_cast<int64_t>(k0 + kk) * a.dout + c0 + c]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kDenseK; ++kk) {
      const float w = Ws[kk][col];
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fmaf(Xs[rg * 4 + i][kk], w, acc[i]);
    }
    __syncthreads();
  }
  if (c0 + col >= a.dout) return;
  const float bias = a.b != nullptr ? to_float(static_cast<const TW*>(a.b)[c0 + col]) : 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = r0 + rg * 4 + i;
    if (row >= a.rows) continue;
    float y = acc[i] + bias;
    if (a.relu) y = fmaxf(y, 0.f);
    store_as(static_cast<TY*>(a.Y) + row * a.dout + c0 + col, y);
  }
}

// The same product when there are few rows (Eq. 2: B m of them): 4 rows x 64 columns per block, the sum over k split
// four ways across the block's wavefronts (every load independent of the others), partial sums combined through LDS.
constexpr int kFewRows = 4, kFewMaxDin = 1024;
template <typename TX, typename TW, typename TY>
__global__ __launch_bounds__(256) void dense_few_rows_kernel(DenseArgs a) {
  __shared__ float Xs[kFewRows][kFewMaxDin];
  __shared__ float red[4][kFewRows][kDenseCols];
  const int tid = threadIdx.x, col = tid % kDenseCols, kq = tid / kDenseCols;
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * kFewRows;
  const int c0 = blockIdx.y * kDenseCols, din = a.d1 + a.d2;
  for (int i = tid; i < kFewRows * din; i += 256) {
    const int r = i / din, k = i % din;
    const int64_t row = r0 + r;
    float v = 0.f;
    if (row < a.rows) {
      v = k < a.d1 ? to_float(static_cast<const TX*>(a.X1)[(row % a.x1_rows) * a.d1 + k])
                   : to_float(static_cast<const TX*>(a.X2)[(row / a.x2_rows_per) * a.d2 + (k - a.d1)]);
    }
    Xs[r][k] = v;
  }
  __syncthreads();
  float acc[kFewRows] = {0.f, 0.f, 0.f, 0.f};
  if (c0 + col < a.dout) {
    const TW* wcol = static_cast<const TW*>(a.W) + c0 + col;
#pragma unroll 8
    for (int k = kq; k < din; k += 4) {
      const float w = to_float(wcol[static_cast<int64_t>(k) * a.dout]);
#pragma unroll
      for (int r = 0; r < kFewRows; ++r) acc[r] = fmaf(Xs[r][k], w, acc[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < kFewRows; ++r) red[kq][r][col] = acc[r];
  __syncthreads();
  // thread (kq, col) finishes row kq
  if (c0 + col >= a.dout || r0 + kq >= a.rows) return;
  float y = red[0][kq][col] + red[1][kq][col] + red[2][kq][col] + red[3][kq][col];
  y += a.b != nullptr ? to_float(static_cast<const TW*>(a.b)[c0 + col]) : 0.f;
  if (a.relu) y = fmaxf(y, 0.f);
  store_as(static_cast<TY*>(a.Y) + (r0 + kq) * a.dout + c0 + col, y);
}

// Few rows and bf16 weights whose rows can be read 16 bytes at a time (d_out a multiple of 8, W 16-byte aligned): a
// thread owns 8 adjacent columns and every 32nd k.  These kernels are chains of memory latencies (Eq. 2 is two of them
// per request), so every load is independent of every other and is issued before the first is used: the rows of X
// through a selected address instead of a test per element (a test makes each load wait for the one before), the
// weights in batches of 16 loads with the index clamped and the out-of-range terms zeroed on the X side.
constexpr int kVecKGroups = 32, kVecBatch = 16;
template <typename TX, typename TY>
__global__ __launch_bounds__(256) void dense_few_rows_vec_kernel(DenseArgs a) {
  __shared__ float Xs[kFewRows][kFewMaxDin];
  __shared__ float red[kVecKGroups][kFewRows * kDenseCols + 1];  // (odd pitch: the k-groups spread over the banks)
  const int tid = threadIdx.x, cg = tid % 8, kq = tid / 8;
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * kFewRows;
  const int c0 = blockIdx.y * kDenseCols + 8 * cg, din = a.d1 + a.d2;
  const int cc = min(c0, a.dout - 8);  // columns past d_out are computed on the last valid ones and not stored
  const bf16_t* W = static_cast<const bf16_t*>(a.W);
  bf16x8 w[kVecBatch];
#pragma unroll
  for (int j = 0; j < kVecBatch; ++j)
    w[j] = *reinterpret_cast<const bf16x8*>(W + static_cast<int64_t>(min(kq + kVecKGroups * j, din - 1)) * a.dout + cc);
  for (int base = 0; base < kFewRows * din; base += 4 * 256) {
    TX v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = min(base + j * 256 + tid, kFewRows * din - 1), k = i % din;
      const int64_t row = min(r0 + i / din, a.rows - 1);
      const TX* src = k < a.d1 ? static_cast<const TX*>(a.X1) + (row % a.x1_rows) * a.d1 + k
                               : static_cast<const TX*>(a.X2) + (row / a.x2_rows_per) * a.d2 + (k - a.d1);
      v[j] = *src;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = base + j * 256 + tid;
      if (i < kFewRows * din) Xs[i / din][i % din] = r0 + i / din < a.rows ? to_float(v[j]) : 0.f;
    }
  }
  __syncthreads();
  float acc[kFewRows][8];
#pragma unroll
  for (int r = 0; r < kFewRows; ++r)
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[r][t] = 0.f;
  for (int k0 = 0; k0 < din; k0 += kVecKGroups * kVecBatch) {
    if (k0 > 0) {  // (d_in beyond 512: the next batch of weight rows)
#pragma unroll
      for (int j = 0; j < kVecBatch; ++j)
        w[j] = *reinterpret_cast<const bf16x8*>(W + static_cast<int64_t>(min(k0 + kq + kVecKGroups * j, din - 1)) * a.dout + cc);
    }
#pragma unroll
    for (int j = 0; j < kVecBatch; ++j) {
      const int k = k0 + kq + kVecKGroups * j;
      if (k0 + kVecKGroups * j >= din) break;  // uniform
#pragma unroll
      for (int r = 0; r < kFewRows; ++r) {
        const float x = k < din ? Xs[r][min(k, din - 1)] : 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[r][t] = fmaf(x, static_cast<float>(w[j][t]), acc[r][t]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < kFewRows; ++r)
#pragma unroll
    for (int t = 0; t < 8; ++t) red[kq][r * kDenseCols + 8 * cg + t] = acc[r][t];
  __syncthreads();
  // thread (r, col) finishes one output
  const int r = tid / kDenseCols, col = blockIdx.y * kDenseCols + tid % kDenseCols;
  if (col >= a.dout || r0 + r >= a.rows) return;
  float y = 0.f;
#pragma unroll 8
  for (int g = 0; g < kVecKGroups; ++g) y += red[g][tid];
  if (a.b != nullptr) y += to_float(static_cast<const bf16_t*>(a.b)[col]);
  if (a.relu) y = fmaxf(y, 0.f);
  store_as(static_cast<TY*>(a.Y) + (r0 + r) * a.dout + col, y);
}

template <typename TX, typename TW, typename TY>
hipError_t launch_dense(const DenseArgs& a, hipStream_t s) {
  if constexpr (std::is_same<TW, bf16_t>::value) {
    if (a.rows <= 2048 && a.d1 + a.d2 <= kFewMaxDin && a.dout >= 8 && a.dout % 8 == 0 &&
        (reinterpret_cast<uintptr_t>(a.W) & 15u) == 0) {
      const dim3 few(static_cast<unsigned>((a.rows + kFewRows - 1) / kFewRows), (a.dout + kDenseCols - 1) / kDenseCols);
      hipLaunchKernelGGL((dense_few_rows_vec_kernel<TX, TY>), few, dim3(256), 0, s, a);
      return hipGetLastError();
    }
  }
  if (a.rows <= 2048 && a.d1 + a.d2 <= kFewMaxDin) {
    const dim3 few(static_cast<unsigned>((a.rows + kFewRows - 1) / kFewRows), (a.dout + kDenseCols - 1) / kDenseCols);
    hipLaunchKernelGGL((dense_few_rows_kernel<TX, TW, TY>), few, dim3(256), 0, s, a);
    return hipGetLastError();
  }
  const dim3 grid(static_cast<unsigned>((a.rows + kDenseRows - 1) / kDenseRows), (a.dout + kDenseCols - 1) / kDenseCols);
  hipLaunchKernelGGL((dense_rows_kernel<TX, TW, TY>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------- interaction network on the matrix cores
// Weight images of the network, written once per call by mlp_pack_kernel (units of bf16x8, one per lane):
//   layer i (d_in x d_out, d_out a multiple of 32): fragment (cb, kk), lane (n, g), slot t = W_i[16kk + k(g, t)][32cb + n],
//   k(g, t) = 8g + t for the first layer (its B operand is read from memory in natural order) and chain_k(g, t) for the
//   others (their B operand is the previous layer's accumulators).
struct MlpArgs {
  const bf16_t* O;        // [rows][D]
  float* scores;          // [rows]
  const bf16x8* img[3];   // hidden layers' weight images
  const bf16_t* bias[3];  // hidden layers' biases
  const bf16_t* w_last;   // [HL] weights of the last affine map
  const bf16_t* b_last;   // [1], nullable
  int64_t rows;
};

template <int D, int H1, int H2, int H3>
__global__ __launch_bounds__(256) void interaction_mlp_kernel(MlpArgs a) {
  constexpr int HL = H3 > 0 ? H3 : (H2 > 0 ? H2 : H1);  // width of the last hidden layer
  constexpr int NB = H1 + H2 + H3 + HL;
  // A 32-column block of a layer's weight image (K/16 fragments of 1 KiB) is the A operand of all four wavefronts.
  // It travels in chunks of at most 16 fragments (16 KiB: a block of the widest layer is two of them): the waves fetch
  // a chunk together, a quarter each, kAhead chunks before its products (one chunk's products are 0.2 us, a fetch
  // from L2 several times that), park it in one of two LDS buffers and read it back from there.
  constexpr int kChunkFrags = 16, kAhead = 3;
  __shared__ bf16x8 stage[2 * kChunkFrags * 64];
  __shared__ __attribute__((aligned(16))) float tab[NB];  // biases of the hidden layers, then the last map's weights
  for (int i = threadIdx.x; i < NB; i += 256) {
    float v;
    if (i < H1) v = a.bias[0] ? to_float(a.bias[0][i]) : 0.f;
    else if (i < H1 + H2) v = a.bias[1] ? to_float(a.bias[1][i - H1]) : 0.f;
    else if (i < H1 + H2 + H3) v = a.bias[2] ? to_float(a.bias[2][i - H1 - H2]) : 0.f;
    else v = to_float(a.w_last[i - H1 - H2 - H3]);
    tab[i] = v;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int64_t row = (static_cast<int64_t>(blockIdx.x) * 4 + wave) * 32 + n;
  // rows past the end are read from the last row and not stored (every wave stays for the barriers)
  const bf16_t* xrow = a.O + (row < a.rows ? row : a.rows - 1) * D + 8 * g;
  bf16x8 xb[D / 16];
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) xb[kk] = *reinterpret_cast<const bf16x8*>(xrow + 16 * kk);

  // one layer: Y^T = W^T X^T block by block; bias and ReLU on the accumulators; the rounded result is the next B operand
  auto layer = [&](auto k_tag, auto out_tag, const bf16x8* img, const bf16x8* in, int bias_at, bf16x8* out, f32x16* keep) {
    constexpr int K = decltype(k_tag)::value, OUT = decltype(out_tag)::value;
    constexpr int KF = K / 16, NCB = OUT / 32;                    // fragments per block, blocks
    constexpr int CH = (KF + kChunkFrags - 1) / kChunkFrags;      // chunks per block
    constexpr int CF = KF / CH;                                   // fragments per chunk (KF is 2, 4, 8, 16 or 32)
    static_assert(CF * CH == KF, "a block is a whole number of equal chunks");
    constexpr int NCH = NCB * CH;                                 // chunks of the layer: chunk c holds fragments c CF ..
    constexpr int PER = (CF + 3) / 4;                             // fragments a wave fetches per chunk
    bf16x8 pre[kAhead][PER];
    auto fetch = [&](int c) {
#pragma unroll
      for (int i = 0; i < PER; ++i)
        if (wave + 4 * i < CF) pre[c % kAhead][i] = img[(c * CF + wave + 4 * i) * 64 + lane];
    };
#pragma unroll
    for (int c = 0; c < kAhead && c < NCH; ++c) fetch(c);
    __syncthreads();  // the previous layer's last chunks have been read by everyone (and tab is written)
    f32x16 acc;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int cb = c / CH, part = c % CH;
      // (the buffer written here was last read two chunks ago, and every wave has passed a barrier since)
      bf16x8* buf = stage + (c & 1) * kChunkFrags * 64;
#pragma unroll
      for (int i = 0; i < PER; ++i)
        if (wave + 4 * i < CF) buf[(wave + 4 * i) * 64 + lane] = pre[c % kAhead][i];
      __syncthreads();
      if (c + kAhead < NCH) fetch(c + kAhead);
      if (part == 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {  // registers 4j .. 4j+3 are columns 32cb + 8j + 4g + 0..3
          const float4 b4 = *reinterpret_cast<const float4*>(&tab[bias_at + 32 * cb + 8 * j + 4 * g]);
          acc[4 * j] = b4.x, acc[4 * j + 1] = b4.y, acc[4 * j + 2] = b4.z, acc[4 * j + 3] = b4.w;
        }
      }
      // every fragment of the chunk is asked for before the first product (one wave per SIMD: nobody else covers the
      // LDS latency, and left alone the compiler reads two fragments ahead and waits for them)
      bf16x8 af[CF];
#pragma unroll
      for (int kk = 0; kk < CF; ++kk) af[kk] = buf[kk * 64 + lane];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < CF; ++kk) acc = mfma32(af[kk], in[part * CF + kk], acc);
      __builtin_amdgcn_sched_barrier(0);
      if (part == CH - 1) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = fmaxf(acc[i], 0.f);
        if (keep != nullptr) {
          keep[cb] = acc;
        } else {
          out[2 * cb] = pack_half(acc, 0);
          out[2 * cb + 1] = pack_half(acc, 1);
        }
      }
    }
  };
  f32x16 last[HL / 32];  // the last hidden layer stays in fp32: one accumulator block per 32 columns
  bf16x8 h1[H1 / 16];
  using std::integral_constant;
  if constexpr (H2 == 0) {
    layer(integral_constant<int, D>{}, integral_constant<int, H1>{}, a.img[0], xb, 0, nullptr, last);
  } else {
    layer(integral_constant<int, D>{}, integral_constant<int, H1>{}, a.img[0], xb, 0, h1, nullptr);
    if constexpr (H3 == 0) {
      layer(integral_constant<int, H1>{}, integral_constant<int, H2>{}, a.img[1], h1, H1, nullptr, last);
    } else {
      bf16x8 h2[H2 / 16];
      layer(integral_constant<int, H1>{}, integral_constant<int, H2>{}, a.img[1], h1, H1, h2, nullptr);
      layer(integral_constant<int, H2>{}, integral_constant<int, H3>{}, a.img[2], h2, H1 + H2, nullptr, last);
    }
  }
  // the logit: a dot product over the last hidden layer (this lane holds the columns 32cb + 8j + 4g + r)
  float s = 0.f;
#pragma unroll
  for (int cb = 0; cb < HL / 32; ++cb)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float4 w4 = *reinterpret_cast<const float4*>(&tab[H1 + H2 + H3 + 32 * cb + 8 * j + 4 * g]);
      s = fmaf(last[cb][4 * j], w4.x, s), s = fmaf(last[cb][4 * j + 1], w4.y, s);
      s = fmaf(last[cb][4 * j + 2], w4.z, s), s = fmaf(last[cb][4 * j + 3], w4.w, s);
    }
  s = pair_sum(s) + (a.b_last != nullptr ? to_float(a.b_last[0]) : 0.f);
  if (g == 0 && row < a.rows) a.scores[row] = s;
}

struct MlpPackArgs {
  const bf16_t* W[3];
  bf16x8* img[3];
  int din[3], dout[3];
  int first_block[4];
};

__global__ __launch_bounds__(256) void mlp_pack_kernel(MlpPackArgs p) {
  int blk = blockIdx.x;
  const int layer = blk >= p.first_block[2] ? 2 : (blk >= p.first_block[1] ? 1 : 0);
  blk -= p.first_block[layer];
  const int din = p.din[layer], dout = p.dout[layer];
  const int idx = blk * 256 + threadIdx.x;  // one 16-byte slot of the image
  if (idx >= din * dout / 8) return;
  const int lane = idx % 64, frag = idx / 64, n = lane & 31, g = lane >> 5;
  const int kk = frag % (din / 16), cb = frag / (din / 16);
  bf16x8 v;
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int k = 16 * kk + (layer == 0 ? 8 * g + t : chain_k(g, t));
    v[t] = __builtin_bit_cast(__bf16, p.W[layer][static_cast<int64_t>(k) * dout + 32 * cb + n].bits);
  }
  p.img[layer][idx] = v;
}

template <int D, int H1, int H2, int H3>
hipError_t launch_mlp(const MlpArgs& a, hipStream_t s) {
  const unsigned grid = static_cast<unsigned>((a.rows + 127) / 128);
  hipLaunchKernelGGL((interaction_mlp_kernel<D, H1, H2, H3>), dim3(grid), dim3(256), 0, s, a);
  return hipGetLastError();
}

// the (D; hidden widths) the matrix-core kernel is built for: Appendix C's three interaction networks on the embedding
// widths this library's matrix-core kernels take
#define LIME_MLP_SHAPES(X) \
  X(256, 512, 128, 64) X(256, 512, 256, 128) X(256, 96, 0, 0) X(128, 512, 128, 64) X(128, 512, 256, 128) X(128, 96, 0, 0) \
  X(64, 512, 128, 64) X(64, 96, 0, 0) X(32, 512, 128, 64) X(32, 512, 256, 128) X(32, 96, 0, 0)

}  // namespace

bool interaction_mlp_on_matrix_cores(int d, int n_maps, const int32_t* widths) {
  if (n_maps < 2 || n_maps > 4 || widths[n_maps - 1] != 1) return false;
  const int h1 = widths[0], h2 = n_maps > 2 ? widths[1] : 0, h3 = n_maps > 3 ? widths[2] : 0;
#define LIME_MLP_MATCH(D_, A_, B_, C_) if (d == D_ && h1 == A_ && h2 == B_ && h3 == C_) return true;
  LIME_MLP_SHAPES(LIME_MLP_MATCH)
#undef LIME_MLP_MATCH
  return false;
}

size_t interaction_mlp_image_bytes(int d, int n_maps, const int32_t* widths) {
  size_t total = 0;
  int din = d;
  for (int i = 0; i + 1 < n_maps; ++i) total += align_up(static_cast<size_t>(din) * widths[i] * 2), din = widths[i];
  return total;
}

hipError_t interaction_mlp_mfma(const void* O, int64_t rows, int d, int n_maps, const int32_t* widths, const void* const* W,
                                const void* const* b, float* scores, void* images, hipStream_t s) {
  MlpPackArgs p{};
  MlpArgs a{};
  a.O = static_cast<const bf16_t*>(O), a.scores = scores, a.rows = rows;
  char* at = static_cast<char*>(images);
  int din = d, blocks = 0;
  for (int i = 0; i < 3; ++i) {
    p.first_block[i] = blocks;
    if (i + 1 < n_maps) {
      p.W[i] = static_cast<const bf16_t*>(W[i]), p.img[i] = reinterpret_cast<bf16x8*>(at);
      p.din[i] = din, p.dout[i] = widths[i];
      a.img[i] = reinterpret_cast<const bf16x8*>(at), a.bias[i] = static_cast<const bf16_t*>(b[i]);
      at += align_up(static_cast<size_t>(din) * widths[i] * 2);
      blocks += (din * widths[i] / 8 + 255) / 256;
      din = widths[i];
    } else {
      p.first_block[i] = 0x7fffffff;
    }
  }
  p.first_block[0] = 0;
  a.w_last = static_cast<const bf16_t*>(W[n_maps - 1]), a.b_last = static_cast<const bf16_t*>(b[n_maps - 1]);
  hipLaunchKernelGGL(mlp_pack_kernel, dim3(blocks), dim3(256), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int h1 = widths[0], h2 = n_maps > 2 ? widths[1] : 0, h3 = n_maps > 3 ? widths[2] : 0;
#define LIME_MLP_LAUNCH(D_, A_, B_, C_) if (d == D_ && h1 == A_ && h2 == B_ && h3 == C_) return launch_mlp<D_, A_, B_, C_>(a, s);
  LIME_MLP_SHAPES(LIME_MLP_LAUNCH)
#undef LIME_MLP_LAUNCH
  return hipErrorInvalidValue;
}

hipError_t layer_norm_rows(const void* X, const void* gamma, const void* beta, float eps, void* Y, int64_t rows, int d,
                           const int32_t* lens, int rows_per_user, int dtype, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  LnArgs a{X, Y, gamma, beta, lens, rows, rows_per_user > 0 ? rows_per_user : 1, d, eps};
  const bool aligned = ((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(Y) | reinterpret_cast<uintptr_t>(gamma) |
                         reinterpret_cast<uintptr_t>(beta)) & 15u) == 0;
  if (dtype == 1 && aligned && d % 8 == 0) {
    const int G = d / 8;
    const unsigned grid = static_cast<unsigned>((rows * G + 255) / 256);
    switch (G) {
#define LIME_LN_CASE(G_) case G_: hipLaunchKernelGGL(layer_norm_bf16_kernel<G_>, dim3(grid), dim3(256), 0, s, a); return hipGetLastError();
      LIME_LN_CASE(4) LIME_LN_CASE(8) LIME_LN_CASE(16) LIME_LN_CASE(32) LIME_LN_CASE(64)
#undef LIME_LN_CASE
      default: break;
    }
  }
  const unsigned grid = static_cast<unsigned>((rows + 3) / 4);
  if (dtype == 1)
    hipLaunchKernelGGL(layer_norm_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(layer_norm_kernel<float>, dim3(grid), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t dense_rows(const Dense& q, hipStream_t s) {
  if (q.rows <= 0) return hipSuccess;
  DenseArgs a{q.X1, q.X2, q.W, q.b, q.Y, q.rows, q.x1_rows > 0 ? q.x1_rows : q.rows, q.x2_rows_per > 0 ? q.x2_rows_per : 1,
              q.d1, q.X2 != nullptr ? q.d2 : 0, q.dout, q.relu ? 1 : 0};
  // (x, w, y) storage: 0 = fp32, 1 = bf16
  const int key = q.x_dtype * 4 + q.w_dtype * 2 + q.y_dtype;
  switch (key) {
    case 0: return launch_dense<float, float, float>(a, s);
    case 2: return launch_dense<float, bf16_t, float>(a, s);
    case 3: return launch_dense<float, bf16_t, bf16_t>(a, s);
    case 6: return launch_dense<bf16_t, bf16_t, float>(a, s);
    case 7: return launch_dense<bf16_t, bf16_t, bf16_t>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace lime
