// Online half of the three-stage inference of Section 3.3: the user-independent attention weights
// phi(T L^t) come from a cache, and the per-candidate interaction is a weighted sum of the personalised
// links, O[c][head a] = sum_i W[c][a][i] V~[i][head a] with V~ = L^P W_V.
//
// Pure streaming: per candidate 2 h m bytes of weights in, 2 d bytes out, 2 m d flops.  One wave per
// head; the head's V~^T (d/h x m) is the stationary MFMA A operand, the weight rows are the B operand.
// A tile is 32 candidates: their weight rows (2 h m bytes each; one contiguous run of memory unless they
// are gathered by id) are copied by all waves together with coalesced 16-byte loads, through a register
// ring that keeps the next tiles in flight, into LDS (padded pitch), where every wave reads its head's
// fragments; the output tile goes back through LDS so that whole row segments are stored, and those stores
// write through the L2 (nobody on the chip reads them again).  Two workgroups share a compute unit.
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
  int B, rows, tiles_per_user, total_tiles;
};

// GATHER: the weight row of candidate (b, c) is row ids[b][c] of a table shared by all users (the
// corpus-wide cache); the ids of a tile are fetched one tile before its weight rows are requested.  An id
// outside the table loads nothing and its output row is written as zeros.
template <int DH, int M, int H, bool GATHER>
__global__ __launch_bounds__(64 * H) void cached_candidates_kernel(CachedArgs a) {
  constexpr int D = DH * H, MB = DH / 32, K3 = M / 16;
  constexpr int CPR = H * M / 8;        // 16-byte chunks per weight row
  constexpr int WB = 2 * H * M;         // bytes per weight row
  constexpr int PITCH = WB + 16;        // LDS row pitch of a weight tile
  constexpr int LW = K3;                // 16-byte loads per lane and tile: 32 CPR / (64 H)
  constexpr int NXS = WB <= 512 ? 2 : 1;  // weight-tile buffers in LDS (one when the rows are long: two barriers per tile)
  constexpr int P = 3;                  // tiles in flight in registers
  constexpr int OCPR = DH / 8, OPITCH = 2 * DH + 16, OLW = DH / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & 63, head = threadIdx.x >> 6;
  const int n = lane & 31, g = lane >> 5;
  unsigned char* otile = lds + NXS * 32 * PITCH + head * 32 * OPITCH;
  const int64_t total_rows = static_cast<int64_t>(a.B) * a.rows;
  const int per_wg = (a.total_tiles + gridDim.x - 1) / gridDim.x;
  const int first = blockIdx.x * per_wg;
  const int last = min(first + per_wg, a.total_tiles);
  if (first >= last) return;  // uniform

  // where this lane's pieces of a tile sit: chunk q = (head LW + j) 64 + lane is chunk q % CPR of row q / CPR
  int rq[LW], cq[LW], ooff[OLW];
#pragma unroll
  for (int j = 0; j < LW; ++j) {
    const int q = (head * LW + j) * 64 + lane;
    rq[j] = q / CPR, cq[j] = q % CPR;
  }
#pragma unroll
  for (int j = 0; j < OLW; ++j) {
    const int o = j * 64 + lane;
    ooff[j] = ((o / OCPR) * D + (o % OCPR) * 8) * 2 + head * DH * 2;
  }
  auto locate = [&](int tile, int& tb, int& tr0) {
    tb = tile / a.tiles_per_user;
    tr0 = (tile - tb * a.tiles_per_user) * 32;
  };
  // the ids of a tile: those of the rows this lane copies, and that of the row it computes (row n)
  auto load_ids = [&](int tile, int (&idj)[LW], int& idn) {
    int tb, tr0;
    locate(tile, tb, tr0);
    const int32_t* src = a.ids + static_cast<int64_t>(tb) * a.rows;
#pragma unroll
    for (int j = 0; j < LW; ++j) idj[j] = src[min(tr0 + rq[j], a.rows - 1)];
    idn = src[min(tr0 + n, a.rows - 1)];
  };
  auto zero = []() {
    bf16x8 v;
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = static_cast<__bf16>(0.f);
    return v;
  };
  auto issue = [&](int tile, const int (&idj)[LW], bf16x8 (&r)[LW]) {
    if constexpr (GATHER) {
#pragma unroll
      for (int j = 0; j < LW; ++j) {
        bf16x8 v = zero();
        if (static_cast<unsigned>(idj[j]) < static_cast<unsigned>(a.n_items))
          v = *reinterpret_cast<const bf16x8*>(a.W + static_cast<int64_t>(idj[j]) * (H * M) + cq[j] * 8);
        r[j] = v;
      }
    } else {
      int tb, tr0;
      locate(tile, tb, tr0);
      // a tile's rows are one contiguous run; rows past a user's last row are read from whatever follows
      // (never stored), rows past the end of the tensor are not read
      const int64_t row0 = static_cast<int64_t>(tb) * a.rows + tr0;
      const unsigned char* base = reinterpret_cast<const unsigned char*>(a.W) + row0 * WB;
      if (row0 + 32 <= total_rows) {  // uniform
#pragma unroll
        for (int j = 0; j < LW; ++j) r[j] = *reinterpret_cast<const bf16x8*>(base + ((head * LW + j) * 64 + lane) * 16);
      } else {
#pragma unroll
        for (int j = 0; j < LW; ++j) {
          bf16x8 v = zero();
          if (row0 + rq[j] < total_rows) v = *reinterpret_cast<const bf16x8*>(base + ((head * LW + j) * 64 + lane) * 16);
          r[j] = v;
        }
      }
    }
  };

  bf16x8 ring[P][LW];
  int ring_idn[P];  // GATHER: the id of row n of the tile in that ring slot
  int idj[LW], idn = 0;
#pragma unroll
  for (int j = 0; j < LW; ++j) idj[j] = 0;
#pragma unroll
  for (int p = 0; p < P; ++p) {
    ring_idn[p] = 0;
    if (first + p < last) {
      if constexpr (GATHER) load_ids(first + p, idj, idn);
      issue(first + p, idj, ring[p]);
      ring_idn[p] = idn;
    }
  }
  if (GATHER && first + P < last) load_ids(first + P, idj, idn);  // of the next tile to request

  bf16x8 va[K3][MB];
  auto load_values = [&](int b) {
    const bf16x8* src = a.VA + b * a.va_user_frags + static_cast<int64_t>(head) * K3 * MB * 64;
#pragma unroll
    for (int kk = 0; kk < K3; ++kk)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) va[kk][mb] = src[(kk * MB + mb) * 64 + lane];
  };
  int cur_user = first / a.tiles_per_user;
  load_values(cur_user);

  for (int base_t = first; base_t < last; base_t += P) {
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int tile = base_t + p;
      if (tile >= last) break;  // uniform over the workgroup
      int b, r0;
      locate(tile, b, r0);
      if (b != cur_user) {
        if (a.va_user_frags != 0) load_values(b);
        cur_user = b;
      }
      unsigned char* buf = lds + (NXS == 2 ? ((tile - first) & 1) : 0) * 32 * PITCH;
#pragma unroll
      for (int j = 0; j < LW; ++j) *reinterpret_cast<bf16x8*>(buf + rq[j] * PITCH + cq[j] * 16) = ring[p][j];
      const int my_id = ring_idn[p];
      // with two buffers a wave arrives here only after it has read the tile before the previous one, which this
      // buffer held; with one, a second barrier follows the reads
      __syncthreads();
      if (tile + P < last) {
        issue(tile + P, idj, ring[p]);
        ring_idn[p] = idn;
        if (GATHER && tile + P + 1 < last) load_ids(tile + P + 1, idj, idn);
      }
      // O^T = V~_a^T W^T: lane (candidate n, g) reads 8 consecutive links of its row per k-step
      bf16x8 pf[K3];
#pragma unroll
      for (int kk = 0; kk < K3; ++kk)
        pf[kk] = *reinterpret_cast<const bf16x8*>(buf + n * PITCH + (head * M + 16 * kk + 8 * g) * 2);
      if (NXS == 1) __syncthreads();
      const bool dead = GATHER && static_cast<unsigned>(my_id) >= static_cast<unsigned>(a.n_items);
#pragma unroll
      for (int ob = 0; ob < MB; ++ob) {
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < K3; ++kk) acc = mfma32(va[kk][ob], pf[kk], acc);
        if (dead) {
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        }
        unsigned char* dst = otile + n * OPITCH + (32 * ob + 16 * g) * 2;
        *reinterpret_cast<bf16x8*>(dst) = pack_half(acc, 0);
        *reinterpret_cast<bf16x8*>(dst + 16) = pack_half(acc, 1);
      }
      // (the wave reads back only what it wrote itself: no barrier)
      bf16x8 ov[OLW];
#pragma unroll
      for (int j = 0; j < OLW; ++j) {
        const int q = j * 64 + lane;
        ov[j] = *reinterpret_cast<const bf16x8*>(otile + (q / OCPR) * OPITCH + (q % OCPR) * 16);
      }
      unsigned char* obase = reinterpret_cast<unsigned char*>(a.O) + (static_cast<int64_t>(b) * a.rows + r0) * (2 * D);
      if (r0 + 32 <= a.rows) {  // uniform: every row of the tile exists
#pragma unroll
        for (int j = 0; j < OLW; ++j) store_through(obase, 32 * 2 * D, ooff[j], ov[j]);
      } else {
#pragma unroll
        for (int j = 0; j < OLW; ++j)
          if (r0 + (j * 64 + lane) / OCPR < a.rows) *reinterpret_cast<bf16x8*>(obase + ooff[j]) = ov[j];
      }
    }
  }
}

template <int DH, int M, int H>
hipError_t launch(const CachedArgs& a, int grid, hipStream_t s) {
  constexpr size_t kPitch = 2 * H * M + 16;
  constexpr size_t kLds = (2 * H * M <= 512 ? 2 : 1) * 32 * kPitch + static_cast<size_t>(H) * 32 * (2 * DH + 16);
  auto gathered = cached_candidates_kernel<DH, M, H, true>;
  auto direct = cached_candidates_kernel<DH, M, H, false>;
  if (kLds > 64 * 1024) {
    static hipError_t attr = [&]() {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gathered), hipFuncAttributeMaxDynamicSharedMemorySize,
                                         static_cast<int>(kLds));
      if (e != hipSuccess) return e;
      return hipFuncSetAttribute(reinterpret_cast<const void*>(direct), hipFuncAttributeMaxDynamicSharedMemorySize,
                                 static_cast<int>(kLds));
    }();
    if (attr != hipSuccess) return attr;
  }
  if (a.ids != nullptr)
    launch_timed(kKernelCachedCandidates, gathered, dim3(grid), dim3(64 * H), kLds, s, a);
  else
    launch_timed(kKernelCachedCandidates, direct, dim3(grid), dim3(64 * H), kLds, s, a);
  return hipGetLastError();
}

template <int DH, int H>
hipError_t dispatch_m(const CachedArgs& a, int m, int grid, hipStream_t s) {
  switch (m) {
    case 32: return launch<DH, 32, H>(a, grid, s);
    case 64: return launch<DH, 64, H>(a, grid, s);
    case 96: return launch<DH, 96, H>(a, grid, s);
    case 128: return launch<DH, 128, H>(a, grid, s);
  }
  return hipErrorInvalidValue;
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
               static_cast<int64_t>(m) * d / 8, q.B, q.C, (q.C + 31) / 32, ((q.C + 31) / 32) * q.B};
  // small register footprint: two workgroups per compute unit cover each other's waits
  const int resident = compute_units() * 2;
  const int grid = a.total_tiles < resident ? a.total_tiles : resident;
  return dh == 32 ? dispatch_h<32>(a, h, m, grid, s) : dispatch_h<64>(a, h, m, grid, s);
}

}  // namespace lime
