// The gated block of the stacked XOR layers (Eq. 8): rows streamed past two stationary weight slices, the two
// products chained through LDS.
#include "mfma.hpp"

namespace lime {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
typedef float f32x4 __attribute__((ext_vector_type(4)));

// The gated block of an XOR layer (Eq. 8) in one pass over the rows:  Y = X + (A * SiLU(X W_U)) W_O.
// One wave per head-sized slice of the d output columns, both weight slices stationary (A operands).  Per tile of
// 32 rows: P^T = W_U^T X^T from the rows' fragments, the gate on the accumulators (a lane owns one row), the gated
// rows Z through LDS (every wave needs all d columns of Z as the B operand of the second product), Y^T = W_O^T Z^T,
// then the residual and, for link rows, the running fp32 sum of the layers' outputs.
struct GatedArgs {
  const bf16_t* X;        // [.][rows][d] the layer's input rows (gate input and residual)
  int64_t x_user_stride;  // elements between users (0 = shared rows)
  const int32_t* lens;    // nullable; rows >= lens[b] count as zeros and are written as zeros
  const bf16x8 *Wu, *Wo;  // weight images
  const bf16_t* A;        // [B][rows][d] attention output of the layer
  bf16_t* Y;              // [B][rows][d] next layer's input; nullable
  const float* sum_in;    // nullable = zero
  float* sum_out;         // nullable
  bf16_t* sum_rounded;    // nullable
  int B, rows, tiles_per_user, total_tiles;
};

template <int DH, int H>
__global__ __launch_bounds__(64 * H) void gated_block_kernel(GatedArgs a) {
  constexpr int D = DH * H, K1 = D / 16, MB = DH / 32;
  constexpr int PITCH = 2 * D + 16;  // bytes; the padding keeps the fragment reads free of bank conflicts
  constexpr int CPR = D / 8;         // 16-byte chunks per row
  constexpr int LW = DH / 16;        // 1 KiB loads per wave and tile: the H waves copy a tile of 32 rows together
  // Three tiles of 32 rows in LDS: the input rows X (fragments of the first product, then the residual), the
  // attention rows A (the gate's other factor; later the staged output rows), the gated rows Z.  Rows travel
  // between memory and LDS in whole 16-byte chunks, row-major and fully coalesced; the accumulator layout (a lane
  // owns a row, four adjacent columns per register quad) only ever touches LDS.
  __shared__ __attribute__((aligned(16))) unsigned char xs[32 * PITCH], as[32 * PITCH], zs[32 * PITCH];
  const int lane = threadIdx.x & 63, head = threadIdx.x >> 6;
  const int n = lane & 31, g = lane >> 5;
  bf16x8 wu[K1][MB], wo[K1][MB];
#pragma unroll
  for (int kk = 0; kk < K1; ++kk)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      wu[kk][mb] = a.Wu[((head * K1 + kk) * MB + mb) * 64 + lane];
      wo[kk][mb] = a.Wo[((head * K1 + kk) * MB + mb) * 64 + lane];
    }
  // this lane's chunks of a tile: (row, chunk) of piece j
  int crow[LW], cchunk[LW];
#pragma unroll
  for (int j = 0; j < LW; ++j) {
    const int q = (head * LW + j) * 64 + lane;
    crow[j] = q / CPR, cchunk[j] = q % CPR;
  }
  bf16x8 rx[LW], ra[LW];
  auto request = [&](int tile) {  // rows at or past the user's length arrive as zeros
    const int b = tile / a.tiles_per_user, r0 = (tile - b * a.tiles_per_user) * 32;
    const int len = a.lens ? min(a.lens[b], a.rows) : a.rows;
#pragma unroll
    for (int j = 0; j < LW; ++j) {
      bf16x8 vx, va;
#pragma unroll
      for (int t = 0; t < 8; ++t) vx[t] = va[t] = static_cast<__bf16>(0.f);
      const int row = r0 + crow[j];
      if (row < len) {
        vx = *reinterpret_cast<const bf16x8*>(a.X + b * a.x_user_stride + static_cast<int64_t>(row) * D + 8 * cchunk[j]);
        va = *reinterpret_cast<const bf16x8*>(a.A + (static_cast<int64_t>(b) * a.rows + row) * D + 8 * cchunk[j]);
      }
      rx[j] = vx, ra[j] = va;
    }
  };
  if (static_cast<int>(blockIdx.x) < a.total_tiles) request(blockIdx.x);
  for (int tile = blockIdx.x; tile < a.total_tiles; tile += gridDim.x) {
    const int b = tile / a.tiles_per_user, r0 = (tile - b * a.tiles_per_user) * 32;
#pragma unroll
    for (int j = 0; j < LW; ++j) {
      *reinterpret_cast<bf16x8*>(xs + crow[j] * PITCH + cchunk[j] * 16) = rx[j];
      *reinterpret_cast<bf16x8*>(as + crow[j] * PITCH + cchunk[j] * 16) = ra[j];
    }
    __syncthreads();
    if (tile + static_cast<int>(gridDim.x) < a.total_tiles) request(tile + gridDim.x);  // in flight during this tile
    // P^T = Wu^T X^T: lane (row n, g), register 4j + r of block mb = column head DH + 32 mb + 8 j + 4 g + r
    f32x16 acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mb][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K1; ++kk)
        acc[mb] = mfma32(wu[kk][mb], *reinterpret_cast<const bf16x8*>(xs + n * PITCH + (16 * kk + 8 * g) * 2), acc[mb]);
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int at = n * PITCH + (head * DH + 32 * mb + 8 * j + 4 * g) * 2;
        const bf16x4 att = *reinterpret_cast<const bf16x4*>(as + at);
        bf16x4 z;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float p = acc[mb][4 * j + r];
          z[r] = static_cast<__bf16>(static_cast<float>(att[r]) * p * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-p * kLog2e)));
        }
        *reinterpret_cast<bf16x4*>(zs + at) = z;
      }
    __syncthreads();  // Z complete; nobody reads the attention rows any more
    f32x16 acc2[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc2[mb][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K1; ++kk)
        acc2[mb] = mfma32(wo[kk][mb], *reinterpret_cast<const bf16x8*>(zs + n * PITCH + (16 * kk + 8 * g) * 2), acc2[mb]);
    }
    const int row = r0 + n;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = head * DH + 32 * mb + 8 * j + 4 * g;
        if (a.Y != nullptr) {  // uniform: the output rows X + Y are staged where the attention rows were
          const bf16x4 xr = *reinterpret_cast<const bf16x4*>(xs + n * PITCH + col * 2);
          bf16x4 y;
#pragma unroll
          for (int r = 0; r < 4; ++r) y[r] = static_cast<__bf16>(static_cast<float>(xr[r]) + acc2[mb][4 * j + r]);
          *reinterpret_cast<bf16x4*>(as + n * PITCH + col * 2) = y;
        }
        if ((a.sum_out != nullptr || a.sum_rounded != nullptr) && row < a.rows) {
          const int64_t at = (static_cast<int64_t>(b) * a.rows + row) * D + col;
          f32x4 t = {0.f, 0.f, 0.f, 0.f};
          if (a.sum_in != nullptr) t = *reinterpret_cast<const f32x4*>(a.sum_in + at);
#pragma unroll
          for (int r = 0; r < 4; ++r) t[r] += acc2[mb][4 * j + r];
          if (a.sum_out != nullptr) *reinterpret_cast<f32x4*>(a.sum_out + at) = t;
          if (a.sum_rounded != nullptr) {
            bf16x4 tr;
#pragma unroll
            for (int r = 0; r < 4; ++r) tr[r] = static_cast<__bf16>(t[r]);
            *reinterpret_cast<bf16x4*>(a.sum_rounded + at) = tr;
          }
        }
      }
    __syncthreads();  // output rows staged; X and Z no longer needed
    if (a.Y != nullptr) {
      // (a row at or past the user's length arrived as zeros and has a zero attention row: its output is zero)
#pragma unroll
      for (int j = 0; j < LW; ++j)
        if (r0 + crow[j] < a.rows)
          *reinterpret_cast<bf16x8*>(a.Y + (static_cast<int64_t>(b) * a.rows + r0 + crow[j]) * D + 8 * cchunk[j]) =
              *reinterpret_cast<const bf16x8*>(as + crow[j] * PITCH + cchunk[j] * 16);
      __syncthreads();  // before the next tile's rows are parked over the staged ones
    }
  }
}

template <int DH, int H>
hipError_t launch_gated(const GatedArgs& p, hipStream_t s) {
  const int resident = (DH * H <= 128 ? 2 : 1) * compute_units();
  hipLaunchKernelGGL((gated_block_kernel<DH, H>), dim3(p.total_tiles < resident ? p.total_tiles : resident), dim3(64 * H), 0, s, p);
  return hipGetLastError();
}

}  // namespace

hipError_t gated_block(const GatedBlock& q, hipStream_t s) {
  if (q.B <= 0 || q.rows <= 0) return hipSuccess;
  const int tiles = (q.rows + 31) / 32;
  GatedArgs p{static_cast<const bf16_t*>(q.X), q.x_user_stride, q.lens, static_cast<const bf16x8*>(q.Wu_image),
              static_cast<const bf16x8*>(q.Wo_image), static_cast<const bf16_t*>(q.A), static_cast<bf16_t*>(q.Y), q.sum_in,
              q.sum_out, static_cast<bf16_t*>(q.sum_rounded), q.B, q.rows, tiles, tiles * q.B};
  const int dh = q.d / q.h;
  if (dh == 32) {
    switch (q.h) {
      case 1: return launch_gated<32, 1>(p, s);
      case 2: return launch_gated<32, 2>(p, s);
      case 4: return launch_gated<32, 4>(p, s);
      case 8: return launch_gated<32, 8>(p, s);
    }
  } else if (dh == 64) {
    switch (q.h) {
      case 1: return launch_gated<64, 1>(p, s);
      case 2: return launch_gated<64, 2>(p, s);
      case 4: return launch_gated<64, 4>(p, s);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace lime
