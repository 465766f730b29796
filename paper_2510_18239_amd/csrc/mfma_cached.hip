// Online half of the three-stage inference of Section 3.3: the user-independent attention weights
// phi(T L^t) come from a cache, and the per-candidate interaction is a weighted sum of the personalised
// links, O[c][head a] = sum_i W[c][a][i] V~[i][head a] with V~ = L^P W_V.
//
// Pure streaming: per candidate 2 h m bytes of weights in, 2 d bytes out, 2 m d flops.  One wave per
// head; the head's V~^T (d/h x m) is the stationary MFMA A operand, the weight rows are the B operand,
// read row-major as stored (lane = candidate, 8 consecutive links).  The kernel is small enough in
// registers that several workgroups share a compute unit, which is what hides the memory latency.
#include "mfma.hpp"

namespace lime {
namespace {

struct CachedArgs {
  const bf16_t* W;   // [B][rows][h][m]
  bf16_t* O;         // [B][rows][d]
  const bf16x8* VA;  // values image, natural k order
  int64_t va_user_frags;
  int rows, tiles_per_user, total_tiles;
};

template <int DH, int M, int H>
__global__ __launch_bounds__(64 * H) void cached_candidates_kernel(CachedArgs a) {
  constexpr int D = DH * H, MB = DH / 32, K3 = M / 16;
  const int lane = threadIdx.x & 63, head = threadIdx.x >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int per_wg = (a.total_tiles + gridDim.x - 1) / gridDim.x;
  const int first = blockIdx.x * per_wg;
  const int last = min(first + per_wg, a.total_tiles);
  if (first >= last) return;

  auto load_weights = [&](int tile, bf16x8 (&p)[K3]) {
    const int b = tile / a.tiles_per_user;
    const int row = min((tile - b * a.tiles_per_user) * 32 + n, a.rows - 1);  // clamped; such columns are not stored
    const bf16_t* src = a.W + ((static_cast<int64_t>(b) * a.rows + row) * H + head) * M + 8 * g;
#pragma unroll
    for (int kk = 0; kk < K3; ++kk) p[kk] = *reinterpret_cast<const bf16x8*>(src + 16 * kk);
  };

  bf16x8 va[K3][MB], pn[K3];
  load_weights(first, pn);
  int cur_user = -1;
  for (int tile = first; tile < last; ++tile) {
    bf16x8 p[K3];
#pragma unroll
    for (int kk = 0; kk < K3; ++kk) p[kk] = pn[kk];
    if (tile + 1 < last) load_weights(tile + 1, pn);
    const int b = tile / a.tiles_per_user;
    const int row = (tile - b * a.tiles_per_user) * 32 + n;
    if (b != cur_user && (cur_user < 0 || a.va_user_frags != 0)) {
      const bf16x8* src = a.VA + b * a.va_user_frags + static_cast<int64_t>(head) * K3 * MB * 64;
#pragma unroll
      for (int kk = 0; kk < K3; ++kk)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) va[kk][mb] = src[(kk * MB + mb) * 64 + lane];
    }
    cur_user = b;
    // O^T = V~_a^T W^T: lane (candidate n, g) gets columns 32 ob + 16 g .. + 15 of the head slice
    bf16_t* orow = a.O + (static_cast<int64_t>(b) * a.rows + row) * D + head * DH + 16 * g;
#pragma unroll
    for (int ob = 0; ob < MB; ++ob) {
      f32x16 acc;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K3; ++kk) acc = mfma32(va[kk][ob], p[kk], acc);
      if (row < a.rows) {
        *reinterpret_cast<bf16x8*>(orow + 32 * ob) = pack_half(acc, 0);
        *reinterpret_cast<bf16x8*>(orow + 32 * ob + 8) = pack_half(acc, 1);
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

template <int DH, int H>
hipError_t dispatch_m(const CachedArgs& a, int m, int grid, hipStream_t s) {
  switch (m) {
    case 32: hipLaunchKernelGGL((cached_candidates_kernel<DH, 32, H>), dim3(grid), dim3(64 * H), 0, s, a); break;
    case 64: hipLaunchKernelGGL((cached_candidates_kernel<DH, 64, H>), dim3(grid), dim3(64 * H), 0, s, a); break;
    case 96: hipLaunchKernelGGL((cached_candidates_kernel<DH, 96, H>), dim3(grid), dim3(64 * H), 0, s, a); break;
    case 128: hipLaunchKernelGGL((cached_candidates_kernel<DH, 128, H>), dim3(grid), dim3(64 * H), 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int DH>
hipError_t dispatch_h(const CachedArgs& a, int h, int m, int grid, hipStream_t s) {
  switch (h) {
    case 1: return dispatch_m<DH, 1>(a, m, grid, s);
    case 2: return dispatch_m<DH, 2>(a, m, grid, s);
    case 4: return dispatch_m<DH, 4>(a, m, grid, s);
    case 8: if (DH == 32) return dispatch_m<32, 8>(a, m, grid, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

size_t cached_candidates_workspace(int B, int d, int m) { return align_up(static_cast<size_t>(B) * m * d * 2); }

hipError_t cached_candidates(const CachedCandidates& q, void* workspace, hipStream_t s) {
  const int d = q.d, h = q.h, m = q.m, dh = d / h;
  PackProject pjob{q.LP, q.Wv, workspace, static_cast<int64_t>(m) * d, q.B, kPackValuesNatural, 1.f};
  hipError_t e = pack_operands(nullptr, 0, &pjob, 1, d, h, m, s);
  if (e != hipSuccess) return e;
  CachedArgs a{static_cast<const bf16_t*>(q.W), static_cast<bf16_t*>(q.O), static_cast<const bf16x8*>(workspace),
               static_cast<int64_t>(m) * d / 8, q.C, (q.C + 31) / 32, ((q.C + 31) / 32) * q.B};
  // small register footprint: several workgroups per compute unit hide the memory latency
  const int resident = compute_units() * 4;
  const int grid = a.total_tiles < resident ? a.total_tiles : resident;
  profile_begin(kKernelCachedCandidates, s);
  e = dh == 32 ? dispatch_h<32>(a, h, m, grid, s) : dispatch_h<64>(a, h, m, grid, s);
  profile_end(kKernelCachedCandidates, s);
  return e;
}

}  // namespace lime
