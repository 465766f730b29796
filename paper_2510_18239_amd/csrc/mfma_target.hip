// Baseline on the matrix cores: full target attention (Eq. 1 with the candidates as queries and
// the history as keys and values; the "MHA skyline" of Section 4.1).  Every candidate attends over
// all N history rows, so the work is O(C N d) per user - the cost LIME avoids.
//
// Two kernels.  (1) project_rows_kernel computes Q~ = T W_Q, K~ = E W_K and V~ = E W_V with the
// weight slices stationary in registers (one wave per head) and writes Q~ row-major and K~, V~ as
// per-tile MFMA fragment images, so that (2) target_attention_kernel, a flash-attention-shaped loop
// over 32-item tiles with the online softmax per query column in the lane's registers, fetches
// every operand with one coalesced 16-byte load per lane:
//   S^T (32 items x 32 q) = K~_tile . Q~^T        O^T (d/h x 32 q) += V~_tile^T . P^T
// History rows at or beyond lens[b] are written as zeros by (1) and masked out of the softmax by (2).
#include "mfma.hpp"

namespace lime {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kOutRows = 0, kOutKeyImage = 1, kOutValueImage = 2;

struct ProjArgs {
  const bf16_t* X;        // [B][rows][d]
  const int32_t* lens;    // nullable; rows >= lens[b] are treated as zeros
  const bf16x8* Wimg;     // weight image
  bf16_t* Y;              // kOutRows: [B][rows][d];  images: [B][tiles][h][...]
  int B, rows, tiles_per_user, total_tiles;
};

// Fragment images per (user, tile of 32 rows, head):
//   keys   [K2][64] : lane (row n, g), slot t = K~[32 tile + n][a dh + 16 kk + 8 g + t]      (A operand, natural k)
//   values [2][MB][64] : lane (col c, g), slot t = V~[32 tile + 16 f + chain_k(g, t)][a dh + 32 ob + c]
template <int DH, int H, int OUT>
__global__ __launch_bounds__(64 * H) void project_rows_kernel(ProjArgs a) {
  constexpr int D = DH * H, K1 = D / 16, MB = DH / 32, K2 = DH / 16;
  const int lane = threadIdx.x & 63, head = threadIdx.x >> 6;
  const int n = lane & 31, g = lane >> 5;
  bf16x8 w[K1][MB];
#pragma unroll
  for (int kk = 0; kk < K1; ++kk)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) w[kk][mb] = a.Wimg[((head * K1 + kk) * MB + mb) * 64 + lane];

  auto load_tile = [&](int tile, bf16x8 (&x)[K1]) {
    const int b = tile / a.tiles_per_user;
    const int row = (tile - b * a.tiles_per_user) * 32 + n;
    const int len = a.lens ? min(a.lens[b], a.rows) : a.rows;
    const bf16_t* xrow = a.X + (static_cast<int64_t>(b) * a.rows + min(row, a.rows - 1)) * D + 8 * g;
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) {
      bf16x8 v;
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = static_cast<__bf16>(0.f);
      if (row < len) v = *reinterpret_cast<const bf16x8*>(xrow + 16 * kk);
      x[kk] = v;
    }
  };

  bf16x8 xn[K1];
  if (static_cast<int>(blockIdx.x) < a.total_tiles) load_tile(blockIdx.x, xn);
  for (int tile = blockIdx.x; tile < a.total_tiles; tile += gridDim.x) {
    bf16x8 x[K1];
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) x[kk] = xn[kk];
    if (tile + static_cast<int>(gridDim.x) < a.total_tiles) load_tile(tile + gridDim.x, xn);
    const int b = tile / a.tiles_per_user, ti = tile - b * a.tiles_per_user;

    f32x16 acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mb][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K1; ++kk)
        acc[mb] = OUT == kOutValueImage ? mfma32(x[kk], w[kk][mb], acc[mb]) : mfma32(w[kk][mb], x[kk], acc[mb]);
    }
    if (OUT == kOutValueImage) {
      // D = X W: lane (column c, g), registers = rows in chained order: the two halves are the fragments
      bf16x8* img = reinterpret_cast<bf16x8*>(a.Y) + (static_cast<int64_t>(tile) * H + head) * 2 * MB * 64;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        img[(0 * MB + mb) * 64 + lane] = pack_half(acc[mb], 0);
        img[(1 * MB + mb) * 64 + lane] = pack_half(acc[mb], 1);
      }
    } else {
      // D = W^T X^T: lane (row n, g), register 4j + r = head column 32 mb + 8 j + 4 g + r
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          bf16x4 v;
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = static_cast<__bf16>(acc[mb][4 * j + r]);
          if (OUT == kOutRows) {
            const int row = ti * 32 + n;
            if (row < a.rows)
              *reinterpret_cast<bf16x4*>(a.Y + (static_cast<int64_t>(b) * a.rows + row) * D + head * DH + 32 * mb +
                                         8 * j + 4 * g) = v;
          } else {
            // head column c = 32 mb + 8 j + 4 g + r belongs to k-step c / 16, lane half (c % 16) / 8, slot c % 8
            const int kk = 2 * mb + (j >> 1);
            bf16_t* frag = a.Y + ((static_cast<int64_t>(tile) * H + head) * K2 + kk) * 64 * 8;
            *reinterpret_cast<bf16x4*>(frag + (32 * (j & 1) + n) * 8 + 4 * g) = v;
          }
        }
    }
  }
}

struct AttnArgs {
  const bf16_t* Q;       // [B][C][d] projected queries
  const bf16x8* Kimg;    // [B][tiles][h][K2][64]
  const bf16x8* Vimg;    // [B][tiles][h][2][MB][64]
  const int32_t* lens;
  bf16_t* O;
  int C, N, tiles_per_user;
  float scale;           // >= 0 (a negative scale is folded into the sign of the packed W_K)
};

template <int DH, int H>
__global__ __launch_bounds__(256) void target_attention_kernel(AttnArgs a) {
  constexpr int D = DH * H, MB = DH / 32, K2 = DH / 16;
  constexpr int QB = 4;  // 32-query blocks per wave: every key / value fragment is used QB times
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int head = blockIdx.y, b = blockIdx.z;
  const int q0 = (blockIdx.x * 4 + wave) * QB * 32;
  if (q0 >= a.C) return;
  const int len = a.lens ? min(a.lens[b], a.N) : a.N;
  const float c = a.scale * kLog2e;

  bf16x8 qf[QB][K2];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int q = min(q0 + 32 * qb + n, a.C - 1);
    const bf16_t* qrow = a.Q + (static_cast<int64_t>(b) * a.C + q) * D + head * DH + 8 * g;
#pragma unroll
    for (int kk = 0; kk < K2; ++kk) qf[qb][kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk);
  }
  f32x16 acc[QB][MB];
  float run_max[QB], run_sum[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    run_max[qb] = -INFINITY;
    run_sum[qb] = 0.f;
#pragma unroll
    for (int ob = 0; ob < MB; ++ob)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[qb][ob][i] = 0.f;
  }

  const int tiles = (len + 31) / 32;
  const bf16x8* kbase = a.Kimg + (static_cast<int64_t>(b) * a.tiles_per_user * H + head) * K2 * 64 + lane;
  const bf16x8* vbase = a.Vimg + (static_cast<int64_t>(b) * a.tiles_per_user * H + head) * 2 * MB * 64 + lane;
  auto load_kv = [&](int t, bf16x8 (&kf)[K2], bf16x8 (&vf)[2][MB]) {
#pragma unroll
    for (int kk = 0; kk < K2; ++kk) kf[kk] = kbase[(static_cast<int64_t>(t) * H * K2 + kk) * 64];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int ob = 0; ob < MB; ++ob) vf[f][ob] = vbase[(static_cast<int64_t>(t) * H * 2 * MB + f * MB + ob) * 64];
  };
  bf16x8 kn[K2], vn[2][MB];
  if (tiles > 0) load_kv(0, kn, vn);

  for (int t = 0; t < tiles; ++t) {
    bf16x8 kf[K2], vf[2][MB];
#pragma unroll
    for (int kk = 0; kk < K2; ++kk) kf[kk] = kn[kk];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int ob = 0; ob < MB; ++ob) vf[f][ob] = vn[f][ob];
    if (t + 1 < tiles) load_kv(t + 1, kn, vn);
    const int i0 = t * 32;
    const bool ragged = i0 + 32 > len;  // uniform: only the user's last tile can hold masked items

#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      f32x16 sc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sc[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K2; ++kk) sc = mfma32(kf[kk], qf[qb][kk], sc);
      // register 4j + r of this lane is item i0 + 8j + 4g + r of query column n
      if (ragged) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (i0 + 8 * (i >> 2) + 4 * g + (i & 3) >= len) sc[i] = -INFINITY;
      }
      float tmax = sc[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, sc[i]);
      tmax = pair_max(tmax);
      const float new_max = fmaxf(run_max[qb], tmax);  // finite: the tile holds at least one valid item
      const float alpha = run_max[qb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((run_max[qb] - new_max) * c);
      const float shift = -new_max * c;
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        // a masked logit is -inf; the explicit select keeps it at weight 0 even for scale = 0
        const float pr = __builtin_amdgcn_exp2f(fmaf(sc[i], c, shift));
        sc[i] = sc[i] == -INFINITY ? 0.f : pr;
        psum += sc[i];
      }
      run_sum[qb] = run_sum[qb] * alpha + psum;
      run_max[qb] = new_max;
      const bf16x8 p0 = pack_half(sc, 0), p1 = pack_half(sc, 1);
#pragma unroll
      for (int ob = 0; ob < MB; ++ob) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[qb][ob][i] *= alpha;
        acc[qb][ob] = mfma32(vf[0][ob], p0, acc[qb][ob]);
        acc[qb][ob] = mfma32(vf[1][ob], p1, acc[qb][ob]);
      }
    }
  }

  // lane (query n of block qb, g) holds head columns 32 ob + 8 j + 4 g + r in register 4 j + r
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int q = q0 + 32 * qb + n;
    const float total = pair_sum(run_sum[qb]);
    const float inv = tiles > 0 ? 1.f / total : 0.f;
    if (q >= a.C) continue;
    bf16_t* orow = a.O + (static_cast<int64_t>(b) * a.C + q) * D + head * DH + 4 * g;
#pragma unroll
    for (int ob = 0; ob < MB; ++ob)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = static_cast<__bf16>(acc[qb][ob][4 * j + r] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * ob + 8 * j) = v;
      }
  }
}

template <int DH, int H>
hipError_t run(const TargetAttention& q, void* workspace, hipStream_t s) {
  constexpr int D = DH * H;
  const int tiles = (q.N + 31) / 32, ctiles = (q.C + 31) / 32;
  char* ws = static_cast<char*>(workspace);
  const size_t wimg = align_up(static_cast<size_t>(D) * D * 2);
  void* Wq = ws;
  void* Wk = ws + wimg;
  void* Wv = ws + 2 * wimg;
  bf16_t* Qt = reinterpret_cast<bf16_t*>(ws + 3 * wimg);
  const size_t qbytes = align_up(static_cast<size_t>(q.B) * q.C * D * 2);
  const size_t kvbytes = align_up(static_cast<size_t>(q.B) * tiles * 32 * D * 2);
  bf16_t* Kimg = reinterpret_cast<bf16_t*>(ws + 3 * wimg + qbytes);
  bf16_t* Vimg = reinterpret_cast<bf16_t*>(ws + 3 * wimg + qbytes + kvbytes);

  // a negative logit scale becomes an exact sign flip of the packed W_K
  PackWeight wjobs[3] = {{q.Wq, Wq, 1.f}, {q.Wk, Wk, q.scale < 0.f ? -1.f : 1.f}, {q.Wv, Wv, 1.f}};
  hipError_t e = pack_operands(wjobs, 3, nullptr, 0, D, H, 32, s);
  if (e != hipSuccess) return e;

  const int resident = compute_units();
  {
    ProjArgs p{static_cast<const bf16_t*>(q.T), nullptr, static_cast<const bf16x8*>(Wq), Qt, q.B, q.C, ctiles, ctiles * q.B};
    launch_timed(kKernelProjection, project_rows_kernel<DH, H, kOutRows>, dim3(p.total_tiles < resident ? p.total_tiles : resident),
                       dim3(64 * H), 0, s, p);
    ProjArgs k{static_cast<const bf16_t*>(q.E), q.lens, static_cast<const bf16x8*>(Wk), Kimg, q.B, q.N, tiles, tiles * q.B};
    launch_timed(kKernelProjection, project_rows_kernel<DH, H, kOutKeyImage>, dim3(k.total_tiles < resident ? k.total_tiles : resident),
                       dim3(64 * H), 0, s, k);
    k.Wimg = static_cast<const bf16x8*>(Wv), k.Y = Vimg;
    launch_timed(kKernelProjection, project_rows_kernel<DH, H, kOutValueImage>, dim3(k.total_tiles < resident ? k.total_tiles : resident),
                       dim3(64 * H), 0, s, k);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  AttnArgs a{Qt, reinterpret_cast<const bf16x8*>(Kimg), reinterpret_cast<const bf16x8*>(Vimg), q.lens,
             static_cast<bf16_t*>(q.O), q.C, q.N, tiles, fabsf(q.scale)};
  const dim3 grid((q.C + 511) / 512, H, q.B);
  launch_timed(kKernelTargetAttention, target_attention_kernel<DH, H>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

bool target_attention_supported(int d, int h) {
  const int dh = d / h;
  return (dh == 32 || dh == 64) && (h == 1 || h == 2 || h == 4 || h == 8) && d <= 256;
}

size_t target_attention_workspace(int B, int C, int N, int d) {
  const int tiles = (N + 31) / 32;
  return 3 * align_up(static_cast<size_t>(d) * d * 2) + align_up(static_cast<size_t>(B) * C * d * 2) +
         2 * align_up(static_cast<size_t>(B) * tiles * 32 * d * 2);
}

hipError_t target_attention(const TargetAttention& q, void* workspace, hipStream_t s) {
  const int dh = q.d / q.h;
  if (dh == 32) {
    switch (q.h) {
      case 1: return run<32, 1>(q, workspace, s);
      case 2: return run<32, 2>(q, workspace, s);
      case 4: return run<32, 4>(q, workspace, s);
      case 8: return run<32, 8>(q, workspace, s);
    }
  } else if (dh == 64) {
    switch (q.h) {
      case 1: return run<64, 1>(q, workspace, s);
      case 2: return run<64, 2>(q, workspace, s);
      case 4: return run<64, 4>(q, workspace, s);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace lime
