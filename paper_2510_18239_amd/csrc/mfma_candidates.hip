// Candidate-side decoupled attention (Eq. 4) on the matrix cores, and with phi = SiLU/m the
// history-to-links direction O[S] of XORA (Eq. 7).
//
// Design: weights stationary in registers, query rows streamed.  A workgroup has one wavefront
// per head.  Wave a keeps, as MFMA A-operand fragments in its registers, the head-a slices of
// W_Q^T (d/h x d), of the projected keys K~ (m x d/h) and of the projected values V~^T (d/h x m).
// For each tile of 32 query rows it chains three contractions without leaving registers:
//   Q~^T (d/h x 32) = W_Q,a^T  . X^T        X rows are the B operand, read row-major as stored
//   S^T  (m   x 32) = K~_a     . Q~^T       B operand = the accumulators of the first product
//   O^T  (d/h x 32) = V~_a^T   . phi(S)^T   B operand = the accumulators of the second product
// Every lane owns one query row (column of the transposed products), so the softmax over the m
// links is a reduction over the lane's own registers plus one exchange with lane ^ 32.
// A small pack kernel computes K~ = Ksrc Wk and V~ = Vsrc Wv once per call and lays all three
// stationary operands out in fragment order, so the main kernel loads them with 16-byte accesses.
#include "mfma.hpp"

namespace lime {
namespace {

constexpr float kLog2e = 1.4426950408889634f;

// ----------------------------------------------------------------------------- main kernel
struct MainArgs {
  const bf16_t* X;
  bf16_t* O;
  const bf16x8 *WqA, *KA, *VA;
  int64_t ka_user_frags, va_user_frags;  // fragment-image size per user (0 = shared), in bf16x8 units
  const int32_t* row_lens;
  int B, rows, tiles_per_user;
  int64_t total_tiles;
  float scale, inv_norm;
};

template <int DH, int M, int H, int PHI>
__global__ __launch_bounds__(64 * H) void queries_over_links_kernel(MainArgs a) {
  constexpr int D = DH * H;
  constexpr int K1 = D / 16, MB = DH / 32;   // first product: k-steps over d, row blocks over d/h
  constexpr int K2 = DH / 16, LB = M / 32;   // second: k-steps over d/h, row blocks over links
  constexpr int K3 = M / 16;                 // third: k-steps over links, row blocks over d/h (MB)
  const int lane = threadIdx.x & 63, head = threadIdx.x >> 6;
  const int n = lane & 31, g = lane >> 5;

  bf16x8 wq[K1][MB];
#pragma unroll
  for (int kk = 0; kk < K1; ++kk)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) wq[kk][mb] = a.WqA[((head * K1 + kk) * MB + mb) * 64 + lane];

  bf16x8 ka[K2][LB], va[K3][MB];
  int cur_user = -1;

  // The X fragments of the next tile are requested before the current tile is computed, so the
  // memory latency hides behind the MFMA work of the one wavefront a SIMD holds.
  auto x_row_ptr = [&](int64_t tile) {
    const int b = static_cast<int>(tile / a.tiles_per_user);
    const int row = static_cast<int>(tile % a.tiles_per_user) * 32 + n;
    // rows past the end are clamped for the load; their columns of the products are never stored
    return a.X + (static_cast<int64_t>(b) * a.rows + min(row, a.rows - 1)) * D + 8 * g;
  };
  bf16x8 xn[K1];
  if (blockIdx.x < a.total_tiles) {
    const bf16_t* xrow = x_row_ptr(blockIdx.x);
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) xn[kk] = *reinterpret_cast<const bf16x8*>(xrow + 16 * kk);
  }

  for (int64_t tile = blockIdx.x; tile < a.total_tiles; tile += gridDim.x) {
    const int b = static_cast<int>(tile / a.tiles_per_user);
    const int r0 = static_cast<int>(tile % a.tiles_per_user) * 32;
    if (b != cur_user) {
      if (cur_user < 0 || a.ka_user_frags != 0) {
        const bf16x8* src = a.KA + b * a.ka_user_frags + static_cast<int64_t>(head) * K2 * LB * 64;
#pragma unroll
        for (int kk = 0; kk < K2; ++kk)
#pragma unroll
          for (int lb = 0; lb < LB; ++lb) ka[kk][lb] = src[(kk * LB + lb) * 64 + lane];
      }
      if (cur_user < 0 || a.va_user_frags != 0) {
        const bf16x8* src = a.VA + b * a.va_user_frags + static_cast<int64_t>(head) * K3 * MB * 64;
#pragma unroll
        for (int kk = 0; kk < K3; ++kk)
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) va[kk][mb] = src[(kk * MB + mb) * 64 + lane];
      }
      cur_user = b;
    }
    const int row = r0 + n;
    const int rlen = a.row_lens ? min(a.row_lens[b], a.rows) : a.rows;
    bf16x8 x[K1];
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) x[kk] = xn[kk];
    if (tile + gridDim.x < a.total_tiles) {
      const bf16_t* xrow = x_row_ptr(tile + gridDim.x);
#pragma unroll
      for (int kk = 0; kk < K1; ++kk) xn[kk] = *reinterpret_cast<const bf16x8*>(xrow + 16 * kk);
    }

    // Q~^T = Wq_a^T X^T
    f32x16 acc1[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc1[mb][i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) acc1[mb] = mfma32(wq[kk][mb], x[kk], acc1[mb]);
    }
    bf16x8 qf[K2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      qf[2 * mb] = pack_half(acc1[mb], 0);
      qf[2 * mb + 1] = pack_half(acc1[mb], 1);
    }

    // S^T = K~_a Q~^T
    f32x16 acc2[LB];
#pragma unroll
    for (int lb = 0; lb < LB; ++lb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc2[lb][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K2; ++kk) acc2[lb] = mfma32(ka[kk][lb], qf[kk], acc2[lb]);
    }

    // phi over the m links of this lane's query row (the other half of the links sits in lane ^ 32)
    float inv = a.inv_norm;
    if (PHI == kPhiSoftmax) {
      float mx = -INFINITY;
#pragma unroll
      for (int lb = 0; lb < LB; ++lb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          acc2[lb][i] *= a.scale;
          mx = fmaxf(mx, acc2[lb][i]);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      float sum = 0.f;
#pragma unroll
      for (int lb = 0; lb < LB; ++lb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = __builtin_amdgcn_exp2f((acc2[lb][i] - mx) * kLog2e);
          acc2[lb][i] = p;
          sum += p;
        }
      sum += __shfl_xor(sum, 32);
      inv = 1.f / sum;
    } else {
#pragma unroll
      for (int lb = 0; lb < LB; ++lb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float s = acc2[lb][i] * a.scale;
          acc2[lb][i] = s / (1.f + __builtin_amdgcn_exp2f(-s * kLog2e));
        }
    }
    bf16x8 pf[K3];
#pragma unroll
    for (int lb = 0; lb < LB; ++lb) {
      pf[2 * lb] = pack_half(acc2[lb], 0);
      pf[2 * lb + 1] = pack_half(acc2[lb], 1);
    }

    // O^T = V~_a^T phi(S)^T, then the normaliser, then 16 consecutive output columns per lane and block
    bf16_t* orow = a.O + (static_cast<int64_t>(b) * a.rows + row) * D + head * DH + 16 * g;
#pragma unroll
    for (int ob = 0; ob < MB; ++ob) {
      f32x16 acc3;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc3[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K3; ++kk) acc3 = mfma32(va[kk][ob], pf[kk], acc3);
      if (row < a.rows) {
        const bool live = row < rlen;
        bf16x8 lo, hi;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          lo[t] = static_cast<__bf16>(live ? acc3[t] * inv : 0.f);
          hi[t] = static_cast<__bf16>(live ? acc3[8 + t] * inv : 0.f);
        }
        *reinterpret_cast<bf16x8*>(orow + 32 * ob) = lo;
        *reinterpret_cast<bf16x8*>(orow + 32 * ob + 8) = hi;
      }
    }
  }
}

int compute_units() {
  static const int n = [] {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0)
      cu = 256;
    return cu;
  }();
  return n;
}

template <int DH, int M, int H>
hipError_t launch_main(const MainArgs& m, int phi, int grid, hipStream_t s) {
  if (phi == kPhiSoftmax)
    hipLaunchKernelGGL((queries_over_links_kernel<DH, M, H, kPhiSoftmax>), dim3(grid), dim3(64 * H), 0, s, m);
  else
    hipLaunchKernelGGL((queries_over_links_kernel<DH, M, H, kPhiSilu>), dim3(grid), dim3(64 * H), 0, s, m);
  return hipGetLastError();
}

template <int DH, int H>
hipError_t dispatch_m(const MainArgs& m, int links, int phi, int grid, hipStream_t s) {
  switch (links) {
    case 32: return launch_main<DH, 32, H>(m, phi, grid, s);
    case 64: return launch_main<DH, 64, H>(m, phi, grid, s);
    case 96: return launch_main<DH, 96, H>(m, phi, grid, s);
    case 128: return launch_main<DH, 128, H>(m, phi, grid, s);
  }
  return hipErrorInvalidValue;
}

template <int DH>
hipError_t dispatch_h(const MainArgs& m, int h, int links, int phi, int grid, hipStream_t s) {
  switch (h) {
    case 1: return dispatch_m<DH, 1>(m, links, phi, grid, s);
    case 2: return dispatch_m<DH, 2>(m, links, phi, grid, s);
    case 4: return dispatch_m<DH, 4>(m, links, phi, grid, s);
    case 8: if (DH == 32) return dispatch_m<32, 8>(m, links, phi, grid, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

bool queries_over_links_supported(int d, int h, int m) {
  const int dh = d / h;
  if (dh != 32 && dh != 64) return false;
  if (h != 1 && h != 2 && h != 4 && h != 8) return false;
  if (d > 256) return false;
  return m % 32 == 0 && m >= 32 && m <= 128;
}

size_t queries_over_links_workspace(int B, int d, int m, bool k_per_user) {
  const size_t wq = align_up(static_cast<size_t>(d) * d * 2);
  const size_t ka = align_up(static_cast<size_t>(k_per_user ? B : 1) * m * d * 2);
  const size_t va = align_up(static_cast<size_t>(B) * m * d * 2);
  return wq + ka + va;
}

hipError_t queries_over_links(const QueriesOverLinks& q, void* workspace, hipStream_t s) {
  const int d = q.d, h = q.h, m = q.m, dh = d / h;
  const bool k_per_user = q.k_user_stride != 0, v_per_user = q.v_user_stride != 0;
  char* ws = static_cast<char*>(workspace);
  bf16_t* WqA = reinterpret_cast<bf16_t*>(ws);
  bf16_t* KA = reinterpret_cast<bf16_t*>(ws + align_up(static_cast<size_t>(d) * d * 2));
  bf16_t* VA = reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(KA) +
                                         align_up(static_cast<size_t>(k_per_user ? q.B : 1) * m * d * 2));
  PackWeight wjob{q.Wq, WqA};
  PackProject pjobs[2] = {{q.Ksrc, q.Wk, KA, q.k_user_stride, k_per_user ? q.B : 1, kPackKeys},
                          {q.Vsrc, q.Wv, VA, q.v_user_stride, v_per_user ? q.B : 1, kPackValues}};
  hipError_t e = pack_operands(&wjob, 1, pjobs, 2, d, h, m, s);
  if (e != hipSuccess) return e;

  MainArgs a{};
  a.X = static_cast<const bf16_t*>(q.X), a.O = static_cast<bf16_t*>(q.O);
  a.WqA = reinterpret_cast<const bf16x8*>(WqA), a.KA = reinterpret_cast<const bf16x8*>(KA);
  a.VA = reinterpret_cast<const bf16x8*>(VA);
  a.ka_user_frags = k_per_user ? static_cast<int64_t>(m) * d / 8 : 0;
  a.va_user_frags = v_per_user ? static_cast<int64_t>(m) * d / 8 : 0;
  a.row_lens = q.row_lens;
  a.B = q.B, a.rows = q.rows, a.tiles_per_user = (q.rows + 31) / 32;
  a.total_tiles = static_cast<int64_t>(a.tiles_per_user) * q.B;
  a.scale = q.scale, a.inv_norm = 1.f / static_cast<float>(m);
  // one resident workgroup per compute unit when the kernel needs most of the register file,
  // two when its footprint is small (d/h = 32)
  const int64_t resident = static_cast<int64_t>(compute_units()) * (dh == 32 && h <= 4 ? 2 : 1);
  const int grid = static_cast<int>(a.total_tiles < resident ? a.total_tiles : resident);
  profile_begin(kKernelQueriesOverLinks, s);
  e = dh == 32 ? dispatch_h<32>(a, h, m, q.phi, grid, s) : dispatch_h<64>(a, h, m, q.phi, grid, s);
  profile_end(kKernelQueriesOverLinks, s);
  return e;
}

}  // namespace lime
