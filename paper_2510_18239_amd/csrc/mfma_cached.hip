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
  const bf16_t* W;   // [B][rows][h][m], or the table [n_items][h][m] when ids are given
  const int32_t* ids;  // nullable: [B][rows]
  int n_items;
  bf16_t* O;         // [B][rows][d]
  const bf16x8* VA;  // values image, natural k order
  int64_t va_user_frags;
  int rows, tiles_per_user, total_tiles;
};

// GATHER: the weight row of candidate (b, c) is row ids[b][c] of a table shared by all users (the
// corpus-wide cache); the ids of a tile are fetched one tile before its weights.
template <int DH, int M, int H, bool GATHER>
__global__ __launch_bounds__(64 * H) void cached_candidates_kernel(CachedArgs a) {
  constexpr int D = DH * H, MB = DH / 32, K3 = M / 16;
  const int lane = threadIdx.x & 63, head = threadIdx.x >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int per_wg = (a.total_tiles + gridDim.x - 1) / gridDim.x;
  const int first = blockIdx.x * per_wg;
  const int last = min(first + per_wg, a.total_tiles);
  if (first >= last) return;

  auto load_id = [&](int tile) -> int {
    const int b = tile / a.tiles_per_user;
    const int row = min((tile - b * a.tiles_per_user) * 32 + n, a.rows - 1);
    return a.ids[static_cast<int64_t>(b) * a.rows + row];
  };
  // `id` is used by the gathering variant only; an id outside the table reads row 0 and is zeroed at the store
  auto load_weights = [&](int tile, int id, bf16x8 (&p)[K3]) {
    const int b = tile / a.tiles_per_user;
    const int row = min((tile - b * a.tiles_per_user) * 32 + n, a.rows - 1);  // clamped; such columns are not stored
    const int64_t wrow = GATHER ? (static_cast<unsigned>(id) < static_cast<unsigned>(a.n_items) ? id : 0)
                                : static_cast<int64_t>(b) * a.rows + row;
    const bf16_t* src = a.W + (wrow * H + head) * M + 8 * g;
#pragma unroll
    for (int kk = 0; kk < K3; ++kk) p[kk] = *reinterpret_cast<const bf16x8*>(src + 16 * kk);
  };

  bf16x8 va[K3][MB], pn[K3];
  int id_next = GATHER ? load_id(first) : 0;  // id of the tile whose weights are in flight
  load_weights(first, id_next, pn);
  int id_ahead = GATHER && first + 1 < last ? load_id(first + 1) : 0;
  int cur_user = -1;
  for (int tile = first; tile < last; ++tile) {
    bf16x8 p[K3];
#pragma unroll
    for (int kk = 0; kk < K3; ++kk) p[kk] = pn[kk];
    const int id = id_next;
    if (tile + 1 < last) {
      id_next = id_ahead;
      load_weights(tile + 1, id_next, pn);
      if (GATHER && tile + 2 < last) id_ahead = load_id(tile + 2);
    }
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
      if (GATHER && static_cast<unsigned>(id) >= static_cast<unsigned>(a.n_items)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
      }
      if (row < a.rows) {
        *reinterpret_cast<bf16x8*>(orow + 32 * ob) = pack_half(acc, 0);
        *reinterpret_cast<bf16x8*>(orow + 32 * ob + 8) = pack_half(acc, 1);
      }
    }
  }
}

template <int DH, int M, int H>
void launch(const CachedArgs& a, int grid, hipStream_t s) {
  if (a.ids != nullptr)
    launch_timed(kKernelCachedCandidates, cached_candidates_kernel<DH, M, H, true>, dim3(grid), dim3(64 * H), 0, s, a);
  else
    launch_timed(kKernelCachedCandidates, cached_candidates_kernel<DH, M, H, false>, dim3(grid), dim3(64 * H), 0, s, a);
}

template <int DH, int H>
hipError_t dispatch_m(const CachedArgs& a, int m, int grid, hipStream_t s) {
  switch (m) {
    case 32: launch<DH, 32, H>(a, grid, s); break;
    case 64: launch<DH, 64, H>(a, grid, s); break;
    case 96: launch<DH, 96, H>(a, grid, s); break;
    case 128: launch<DH, 128, H>(a, grid, s); break;
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
  CachedArgs a{static_cast<const bf16_t*>(q.W), q.ids, q.n_items, static_cast<bf16_t*>(q.O), static_cast<const bf16x8*>(workspace),
               static_cast<int64_t>(m) * d / 8, q.C, (q.C + 31) / 32, ((q.C + 31) / 32) * q.B};
  // small register footprint: several workgroups per compute unit hide the memory latency
  const int resident = compute_units() * 4;
  const int grid = a.total_tiles < resident ? a.total_tiles : resident;
  e = dh == 32 ? dispatch_h<32>(a, h, m, grid, s) : dispatch_h<64>(a, h, m, grid, s);
  return e;
}

}  // namespace lime
