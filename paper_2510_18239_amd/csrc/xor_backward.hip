// Backward pass of one XORA layer with respect to its projected inputs (Appendix H.2), with the attention matrices
// recomputed tile by tile (nothing of size N x m is stored): a matrix-core form for bf16 storage and a form in fp32
// arithmetic on the vector ALUs for everything else.
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
#include <algorithm>

#include "common.hpp"
#include "mfma.hpp"

namespace lime {
namespace {

constexpr int kOwn = 32;    // rows of X per workgroup
constexpr int kMaxDh = 64;  // widest head

struct SideArgs {
  const void *qx, *kx, *vx, *gx;  // [B][rows_x][d]; gx nullable (no upstream gradient for O[X])
  const void *qy, *ky, *vy, *gy;  // [B][rows_y][d]; gy nullable
  void *dq, *dk, *dv;             // [B][rows_x][d], storage type: written when chunks == 1
  float* partial;                 // [B][chunks][3][rows_x][d]: written when chunks > 1
  const int32_t* lens;            // valid history rows per user, nullable = all
  int own_is_history;             // which side the lengths apply to
  int rows_x, rows_y, d, dh, chunks, chunk_rows;  // chunk_rows: rows of Y per chunk, a multiple of the step
  float scale;
};

// sigmoid with the hardware's exp2 and reciprocal (about one ulp each); SiLU(x) = x s, SiLU'(x) = s (1 + x (1 - s))
__device__ __forceinline__ float sigmoid_f(float x) {
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}
__device__ __forceinline__ float silu_derivative_from(float x, float s) { return s * fmaf(x, 1.f - s, 1.f); }
__device__ __forceinline__ float dot4(const float4& a, const float4& b, float c) {
  return fmaf(a.w, b.w, fmaf(a.z, b.z, fmaf(a.y, b.y, fmaf(a.x, b.x, c))));
}

// DHM: the head width the LDS tiles are sized for (d/h <= DHM); OTHER: rows of Y per step (32, or 16 where the
// wider head would not leave room).  The tiles are stored transposed, [column of the head][row], so that a thread
// reads two adjacent rows (dot-product step) or four adjacent rows of Y (accumulation step) with one LDS access:
// the vector ALUs, not the LDS, then set the pace.
template <typename T, int DHM, int OTHER>
__global__ __launch_bounds__(256) void xor_backward_side_kernel(SideArgs a) {
  constexpr int SX = kOwn + 4, SY = OTHER + 4;  // row pitches: multiples of four words (16-byte reads), not of 32
  constexpr int CP = OTHER / 16;                // columns of the pair tile per thread in the dot-product step
  constexpr int J = DHM / 8;                    // output columns per thread
  __shared__ __align__(16) float own[4][DHM][SX];    // q, k, v, g of the block's rows of X (head slice)
  __shared__ __align__(16) float other[4][DHM][SY];  // q, k, v, g of the current rows of Y
  __shared__ __align__(16) float p1[kOwn][SY], e1[kOwn][SY], e2[kOwn][SY];
  const int tid = threadIdx.x, dh = a.dh, d = a.d;
  const int blocks_x = (a.rows_x + kOwn - 1) / kOwn;
  const int xb = blockIdx.x % blocks_x, chunk = blockIdx.x / blocks_x, head = blockIdx.y, b = blockIdx.z;
  const int hist_rows = a.own_is_history ? a.rows_x : a.rows_y;
  const int len = a.lens ? min(max(a.lens[b], 0), hist_rows) : hist_rows;
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
  // (indexed by the tile's compile-time width, so that the index arithmetic is shifts; columns past d/h are skipped)
  for (int i = tid; i < 4 * kOwn * DHM; i += 256) {
    const int w = i / (kOwn * DHM), r = (i / DHM) % kOwn, t = i % DHM;
    if (t < dh)
      own[w][t][r] = (own_src[w] != nullptr && r0 + r < valid_x) ? to_float(own_src[w][x_base + static_cast<int64_t>(r) * d + t]) : 0.f;
  }
  // accumulation step: thread (r, tc) owns columns tc, tc + 8, ... of row r of the three outputs
  const int r = tid / 8, tc = tid % 8;
  float dq[J], dk[J], dv[J];
#pragma unroll
  for (int j = 0; j < J; ++j) dq[j] = dk[j] = dv[j] = 0.f;
  // dot-product step: thread owns rows pr0, pr0 + 1 and columns pc0 .. pc0 + CP - 1 of the kOwn x OTHER pair tile
  const int pr0 = 2 * (tid / 16), pc0 = CP * (tid % 16);

  const int c_begin = chunk * a.chunk_rows, c_end = min(c_begin + a.chunk_rows, valid_y);
  // The rows of Y for the next step are asked for before the current step is computed and parked in LDS after it:
  // a step's loads are in flight while the previous one keeps the vector ALUs busy.
  constexpr int kLoads = 4 * OTHER * DHM / 256;
  float ahead[kLoads];
  auto ask = [&](int c0) {
    const int64_t y_base = (static_cast<int64_t>(b) * a.rows_y + c0) * d + head * dh;
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const int i = tid + 256 * k;
      const int w = i / (OTHER * DHM), c = (i / DHM) % OTHER, t = i % DHM;
      ahead[k] = (t < dh && other_src[w] != nullptr && c0 + c < c_end)
                     ? to_float(other_src[w][y_base + static_cast<int64_t>(c) * d + t]) : 0.f;
    }
  };
  if (c_begin < c_end) ask(c_begin);
  for (int c0 = c_begin; c0 < c_end; c0 += OTHER) {
    __syncthreads();  // the previous step is done with `other`, p1, e1, e2 (and `own` is complete)
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const int i = tid + 256 * k;
      other[i / (OTHER * DHM)][i % DHM][(i / DHM) % OTHER] = ahead[k];
    }
    __syncthreads();
    if (c0 + OTHER < c_end) ask(c0 + OTHER);
    float z1[2][CP], w1[2][CP], z2[2][CP], w2[2][CP];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < CP; ++j) z1[i][j] = w1[i][j] = z2[i][j] = w2[i][j] = 0.f;
    for (int t = 0; t < dh; ++t) {
      const float2 qx = *reinterpret_cast<const float2*>(&own[0][t][pr0]);
      const float2 kx = *reinterpret_cast<const float2*>(&own[1][t][pr0]);
      const float2 vx = *reinterpret_cast<const float2*>(&own[2][t][pr0]);
      const float2 gx = *reinterpret_cast<const float2*>(&own[3][t][pr0]);
      const float xq[2] = {qx.x, qx.y}, xk[2] = {kx.x, kx.y}, xv[2] = {vx.x, vx.y}, xg[2] = {gx.x, gx.y};
#pragma unroll
      for (int j = 0; j < CP; ++j) {
        const float qy = other[0][t][pc0 + j], ky = other[1][t][pc0 + j], vy = other[2][t][pc0 + j],
                    gy = other[3][t][pc0 + j];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          z1[i][j] = fmaf(qy, xk[i], z1[i][j]);  // <Q[Y]_c, K[X]_r>
          w1[i][j] = fmaf(gy, xv[i], w1[i][j]);  // <G[Y]_c, V[X]_r>
          z2[i][j] = fmaf(xq[i], ky, z2[i][j]);  // <Q[X]_r, K[Y]_c>
          w2[i][j] = fmaf(xg[i], vy, w2[i][j]);  // <G[X]_r, V[Y]_c>
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < CP; ++j) {
        const float s1 = z1[i][j] * a.scale, s2 = z2[i][j] * a.scale;
        const bool live = r0 + pr0 + i < valid_x && c0 + pc0 + j < c_end;
        const float g1 = sigmoid_f(s1), g2 = sigmoid_f(s2);
        p1[pr0 + i][pc0 + j] = live ? s1 * g1 * inv_nx : 0.f;
        e1[pr0 + i][pc0 + j] = live ? w1[i][j] * silu_derivative_from(s1, g1) * inv_nx * a.scale : 0.f;
        e2[pr0 + i][pc0 + j] = live ? w2[i][j] * silu_derivative_from(s2, g2) * inv_ny * a.scale : 0.f;
      }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < OTHER; c += 4) {
      const float4 p = *reinterpret_cast<const float4*>(&p1[r][c]);
      const float4 f1 = *reinterpret_cast<const float4*>(&e1[r][c]);
      const float4 f2 = *reinterpret_cast<const float4*>(&e2[r][c]);
#pragma unroll
      for (int j = 0; j < J; ++j) {
        const int t = tc + 8 * j;
        if (t < dh) {
          dv[j] = dot4(p, *reinterpret_cast<const float4*>(&other[3][t][c]), dv[j]);
          dk[j] = dot4(f1, *reinterpret_cast<const float4*>(&other[0][t][c]), dk[j]);
          dq[j] = dot4(f2, *reinterpret_cast<const float4*>(&other[1][t][c]), dq[j]);
        }
      }
    }
  }
  if (r0 + r >= a.rows_x) return;
  const int64_t row = static_cast<int64_t>(b) * a.rows_x + r0 + r;
#pragma unroll
  for (int j = 0; j < J; ++j) {
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

// The same step on the matrix cores (bf16 storage, d/h = 32 or 64): every contraction is a 32 x 32 x 16 MFMA.
// Each of the workgroup's four waves takes its own 32 rows of Y per step and runs the whole step in registers:
//   1. the four dot-product tiles, transposed: D[c][r] = <Y-tensor_c, X-tensor_r>, A operand = rows of Y, B operand =
//      rows of X, both read row-major with the summed head columns contiguous.  All four land in the same accumulator
//      layout (lane = row r of X, registers = rows c of Y), so p1, e1, e2 are computed register by register;
//   2. an accumulator block is, as it stands, the B operand of a product that sums over its rows (chained order):
//      dV[X]^T[t][r] += sum_c G[Y]^T[t][c] p1[c][r], likewise dK with Q[Y] and e1, dQ with K[Y] and e2.  The A operand
//      is the transposed Y tensor in the same chained order, read from a transposed copy the wave parks in its own
//      piece of LDS (no barrier: a wave reads back only what it wrote itself);
//   3. after the last step the four waves' sums meet in LDS in wave order and are stored.
// With OWN_PER_WAVE (many rows of X, few of Y: the history side) each wave instead takes its own 32 rows of X, walks
// all of Y itself and stores its accumulators directly: no sums to combine.
// Rows that are not valid are loaded as zeros, which makes every term they touch zero (SiLU(0) = 0, and e1, e2 carry
// a dot product with the zero row).
// The transposed copy is written one bf16 at a time and read back four at a time: both through types that may alias
// anything, so that the compiler keeps the order of a wave's stores and loads.
typedef __bf16 __attribute__((may_alias)) bf16_any;
typedef bf16x4 __attribute__((may_alias)) bf16x4_any;
constexpr int kMfmaStep = 128;  // rows of Y per workgroup step: 32 per wave
template <int DH, bool OWN_PER_WAVE>
__global__ __launch_bounds__(256, (DH == 32 ? 2 : 1)) void xor_backward_side_mfma_kernel(SideArgs a) {
  constexpr int KS = DH / 16, TT = DH / 32, PITCH = 36;  // PITCH: bf16 per row of the transposed copy (8-byte reads)
  constexpr int kWaveTile = 3 * DH * PITCH;              // bf16: transposed Q[Y], K[Y], G[Y] of one wave
  constexpr int kRed = 3 * TT * 16 * 64;                 // floats: one wave's output accumulators
  constexpr size_t kBytes = sizeof(float) * kRed > 2 * 4 * kWaveTile ? sizeof(float) * kRed : 2 * 4 * kWaveTile;
  __shared__ __align__(16) unsigned char smem[kBytes];
  const int tid = threadIdx.x, wv = tid / 64, lane = tid % 64, n = lane % 32, g = lane / 32, d = a.d;
  const int own_rows = OWN_PER_WAVE ? 4 * kOwn : kOwn;  // rows of X per workgroup
  const int blocks_x = (a.rows_x + own_rows - 1) / own_rows;
  const int xb = blockIdx.x % blocks_x, chunk = blockIdx.x / blocks_x, head = blockIdx.y, b = blockIdx.z;
  const int hist_rows = a.own_is_history ? a.rows_x : a.rows_y;
  const int len = a.lens ? min(max(a.lens[b], 0), hist_rows) : hist_rows;
  const int valid_x = a.own_is_history ? len : a.rows_x, valid_y = a.own_is_history ? a.rows_y : len;
  const float inv_nx = valid_x > 0 ? 1.f / static_cast<float>(valid_x) : 0.f;
  const float inv_ny = valid_y > 0 ? 1.f / static_cast<float>(valid_y) : 0.f;
  const int r0 = xb * own_rows + (OWN_PER_WAVE ? wv * kOwn : 0);
  bf16x8 zero;
#pragma unroll
  for (int t = 0; t < 8; ++t) zero[t] = static_cast<__bf16>(0.f);
  // A 32-row tile of a row-major tensor (head slice) is fetched row-contiguous - KS loads of 16 bytes per lane, DH/8
  // lanes per row, so that a load touches few cache lines - and turned into operand fragments (lane (n, g) holds
  // columns 16ks + 8g .. + 7 of row n) through the wave's piece of LDS.  Rows at or past `limit` count as zeros.
  constexpr int P2 = DH + 8, CPR = DH / 8;  // bf16 per staged row; 16-byte pieces per row
  typedef bf16x8 __attribute__((may_alias)) bf16x8_any;
  auto fetch = [&](const void* base, int rows, int row0, int limit, bf16x8 (&piece)[KS]) {
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      const int idx = lane + 64 * i, row = row0 + idx / CPR;
      piece[i] = (base == nullptr || row >= limit) ? zero
                 : *reinterpret_cast<const bf16x8*>(static_cast<const bf16_t*>(base) +
                                                    (static_cast<int64_t>(b) * rows + row) * d + head * DH + 8 * (idx % CPR));
    }
  };
  bf16_any* yt = reinterpret_cast<bf16_any*>(smem) + wv * kWaveTile;  // [3][DH][PITCH]: Q[Y]^T, K[Y]^T, G[Y]^T
  auto to_fragments = [&](const bf16x8 (&piece)[KS], bf16x8 (&fr)[KS]) {
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      const int idx = lane + 64 * i;
      *reinterpret_cast<bf16x8_any*>(yt + (idx / CPR) * P2 + 8 * (idx % CPR)) = piece[i];
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fr[ks] = *reinterpret_cast<const bf16x8_any*>(yt + n * P2 + 16 * ks + 8 * g);
  };
  // the block's rows of X as B operands (lane = row r0 + n): q, k, v, g
  bf16x8 xq[KS], xk[KS], xv[KS], xg[KS];
  {
    bf16x8 pq[KS], pk[KS], pv[KS], pg[KS];
    fetch(a.qx, a.rows_x, r0, valid_x, pq), fetch(a.kx, a.rows_x, r0, valid_x, pk);
    fetch(a.vx, a.rows_x, r0, valid_x, pv), fetch(a.gx, a.rows_x, r0, valid_x, pg);
    to_fragments(pq, xq), to_fragments(pk, xk), to_fragments(pv, xv), to_fragments(pg, xg);
  }
  f32x16 acc[3][TT];  // dV^T, dK^T, dQ^T: lane = row r0 + n, register 4j + rr = head column 32tt + 8j + 4g + rr
#pragma unroll
  for (int o = 0; o < 3; ++o)
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[o][tt][i] = 0.f;
  const int c_begin = chunk * a.chunk_rows, c_end = min(c_begin + a.chunk_rows, valid_y);
  const int c_first = c_begin + (OWN_PER_WAVE ? 0 : 32 * wv), c_step = OWN_PER_WAVE ? 32 : kMfmaStep;
  // the wave's next 32 rows of Y (row-contiguous pieces, made into A operands when their step starts): asked for one
  // step ahead
  bf16x8 nq[KS], nk[KS], nv[KS], ng[KS];
  auto ask = [&](int c0) {
    fetch(a.qy, a.rows_y, c0, c_end, nq), fetch(a.ky, a.rows_y, c0, c_end, nk);
    fetch(a.vy, a.rows_y, c0, c_end, nv), fetch(a.gy, a.rows_y, c0, c_end, ng);
  };
  if (c_first < c_end) ask(c_first);
  for (int c0 = c_first; c0 < c_end; c0 += c_step) {
    bf16x8 yq[KS], yk[KS], yv[KS], yg[KS];
    to_fragments(nq, yq), to_fragments(nk, yk), to_fragments(nv, yv), to_fragments(ng, yg);
    if (c0 + c_step < c_end) ask(c0 + c_step);
    f32x16 z1, w1, z2, w2;
#pragma unroll
    for (int i = 0; i < 16; ++i) z1[i] = w1[i] = z2[i] = w2[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      z1 = mfma32(yq[ks], xk[ks], z1);  // <Q[Y]_c, K[X]_r>
      w1 = mfma32(yg[ks], xv[ks], w1);  // <G[Y]_c, V[X]_r>
      z2 = mfma32(yk[ks], xq[ks], z2);  // <K[Y]_c, Q[X]_r>
      w2 = mfma32(yv[ks], xg[ks], w2);  // <V[Y]_c, G[X]_r>
      // the transposed copy: column 16ks + 8g + t of row c0 + n goes to [column][n]
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int col = 16 * ks + 8 * g + t;
        yt[(0 * DH + col) * PITCH + n] = yq[ks][t];
        yt[(1 * DH + col) * PITCH + n] = yk[ks][t];
        yt[(2 * DH + col) * PITCH + n] = yg[ks][t];
      }
    }
    // phi and phi' register by register: z1 becomes p1, w1 becomes e1, w2 becomes e2
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float s1 = z1[i] * a.scale, s2 = z2[i] * a.scale;
      const float g1 = sigmoid_f(s1), g2 = sigmoid_f(s2);
      z1[i] = s1 * g1 * inv_nx;
      w1[i] = w1[i] * silu_derivative_from(s1, g1) * (inv_nx * a.scale);
      w2[i] = w2[i] * silu_derivative_from(s2, g2) * (inv_ny * a.scale);
    }
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      const bf16x8 bp = pack_half(z1, f), be1 = pack_half(w1, f), be2 = pack_half(w2, f);
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        // slot t of lane (n, g): row c0 + 16f + chain_k(g, t) of Y, head column 32tt + n
        auto chained = [&](int arr) {
          const bf16_any* src = yt + (arr * DH + 32 * tt + n) * PITCH + 16 * f + 4 * g;
          const bf16x4 lo = *reinterpret_cast<const bf16x4_any*>(src), hi = *reinterpret_cast<const bf16x4_any*>(src + 8);
          bf16x8 v;
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] = lo[t], v[4 + t] = hi[t];
          return v;
        };
        acc[0][tt] = mfma32(chained(2), bp, acc[0][tt]);   // dV[X]^T += G[Y]^T p1
        acc[1][tt] = mfma32(chained(0), be1, acc[1][tt]);  // dK[X]^T += Q[Y]^T e1
        acc[2][tt] = mfma32(chained(1), be2, acc[2][tt]);  // dQ[X]^T += K[Y]^T e2
      }
    }
  }
  auto out_of = [&](int which) { return static_cast<bf16_t*>(which == 0 ? a.dq : (which == 1 ? a.dk : a.dv)); };
  const int64_t plane = static_cast<int64_t>(a.rows_x) * d;
  if constexpr (OWN_PER_WAVE) {
    // lane (n, g) holds, for its row r0 + n, head columns 32tt + 8j + 4g .. + 3 in registers 4j .. 4j + 3
    if (a.chunks == 1) {
      // Stored through the wave's piece of LDS, so that a store instruction writes whole head slices of a few rows
      // (16 bytes per lane, four or eight lanes per row) instead of eight bytes in each of 32 rows: the memory
      // pipeline works per cache line touched.
#pragma unroll
      for (int o = 0; o < 3; ++o) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            bf16x4 v;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) v[rr] = static_cast<__bf16>(acc[o][tt][4 * j + rr]);
            *reinterpret_cast<bf16x4_any*>(yt + n * P2 + 32 * tt + 8 * j + 4 * g) = v;
          }
        bf16_t* out = out_of(2 - o);  // accumulators are (dV, dK, dQ); outputs are ordered (dQ, dK, dV)
#pragma unroll
        for (int i = 0; i < 32 * CPR / 64; ++i) {
          const int idx = lane + 64 * i, row = idx / CPR, piece = idx % CPR;
          const bf16x8 v = *reinterpret_cast<const bf16x8_any*>(yt + row * P2 + 8 * piece);
          if (r0 + row < a.rows_x)
            *reinterpret_cast<bf16x8_any*>(out + (static_cast<int64_t>(b) * a.rows_x + r0 + row) * d + head * DH + 8 * piece) = v;
        }
      }
      return;
    }
    if (r0 + n >= a.rows_x) return;
#pragma unroll
    for (int o = 0; o < 3; ++o) {
      const int which = 2 - o;
#pragma unroll
      for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float* dst = a.partial + ((static_cast<int64_t>(b) * a.chunks + chunk) * 3 + which) * plane +
                       static_cast<int64_t>(r0 + n) * d + head * DH + 32 * tt + 8 * j + 4 * g;
          *reinterpret_cast<float4*>(dst) = make_float4(acc[o][tt][4 * j], acc[o][tt][4 * j + 1], acc[o][tt][4 * j + 2],
                                                        acc[o][tt][4 * j + 3]);
        }
    }
    return;
  }
  // the four waves' sums, added in wave order
  float* red = reinterpret_cast<float*>(smem);
  for (int turn = 0; turn < 4; ++turn) {
    __syncthreads();  // (the first one also ends every wave's use of its transposed copy)
    if (wv == turn) {
#pragma unroll
      for (int o = 0; o < 3; ++o)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            float* at = red + ((o * TT + tt) * 16 + i) * 64 + lane;
            *at = turn == 0 ? acc[o][tt][i] : *at + acc[o][tt][i];
          }
    }
  }
  __syncthreads();
  for (int e = tid; e < kRed; e += 256) {
    const int o = e / (TT * 1024), tt = (e / 1024) % TT, i = (e / 64) % 16, l = e % 64;
    const int row = r0 + l % 32, col = 32 * tt + 8 * (i / 4) + 4 * (l / 32) + i % 4;
    if (row >= a.rows_x) continue;
    const int64_t at = (static_cast<int64_t>(b) * a.rows_x + row) * d + head * DH + col;
    const int which = 2 - o;  // accumulators are (dV, dK, dQ); outputs are ordered (dQ, dK, dV)
    if (a.chunks == 1)
      store_as(out_of(which) + at, red[e]);
    else
      a.partial[((static_cast<int64_t>(b) * a.chunks + chunk) * 3 + which) * plane + static_cast<int64_t>(row) * d + head * DH + col] = red[e];
  }
}

// Both sides in one pass (bf16 storage, d/h = 32 or 64, MB blocks of 32 links): the history rows, which are the bulk of the
// operands, are read once, and phi, phi' - an exponential and a reciprocal per logit, the vector ALUs' share, which
// sets the pace of the two-kernel form - are evaluated once per pair instead of once per side.
// A workgroup of eight waves at d/h = 32 with up to 64 links (two per SIMD: one wave's waits for LDS, memory and the
// matrix cores are the other's time to issue; at d/h = 64, and with 96 or 128 links, the links' sums alone are 144 to
// 192 registers and a workgroup is four waves) takes a chunk of the history of one (user, head); each wave walks its own 32-row tiles of it.  The links' operands lie in LDS as
// fragment images, shared by the waves and read where they are used: in registers they would leave no room for a
// second wave.  Per tile:
//   1. its four tensors come straight from memory as operand fragments, asked for while the previous tile's last
//      products run; Q[S], K[S], G[S] are also parked transposed in the wave's piece of LDS;
//   2. per block of 32 links, one direction after the other: a logit tile and a <G, V> tile with the history rows as
//      A operand and the links as B operand (lane = link t, registers = history rows s), phi and phi' register by
//      register, rounded to bf16: p1, e1 (direction O[T]), then p2, e2 (direction O[S]);
//   3. the links' gradients sum over the history rows, which those blocks hold in their registers: p2, e1, e2 are
//      chained B operands as they stand (as in the kernel above), dV[T]^T += G[S]^T p2, dQ[T]^T += K[S]^T e1,
//      dK[T]^T += Q[S]^T e2, accumulated over the wave's whole walk;
//   4. the history rows' gradients sum over the links, the lane index of those blocks: p1, e1, e2 are parked in LDS
//      ([history row][link], one bf16 at a time) and - after the last block of links, or with three and four
//      blocks right away - read back as B operands (lane = history row, eight links per lane) against the links'
//      transposed operands: dV[S]^T += G[T]^T p1^T,
//      dK[S]^T += Q[T]^T e1^T, dQ[S]^T += K[T]^T e2^T; stored through LDS as whole head slices of a few rows.
// The constant factors (scale, 1/n_S, 1/m) are left out of the tiles and applied to the sums.  At the end the waves'
// sums for the links meet in LDS pairwise in a fixed order; chunk sums as above.  The steps of a tile are fenced
// against the instruction scheduler: moved into each other they need more registers than two waves per SIMD leave.
typedef bf16x8 __attribute__((may_alias)) bf16x8_any;
typedef unsigned short __attribute__((may_alias)) u16_any;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
struct FusedArgs {
  const void *qs, *ks, *vs, *gs;  // [B][N][d]; gs nullable (no upstream gradient for O[S])
  const void *qt, *kt, *vt, *gt;  // [B][m][d]
  void *dqs, *dks, *dvs;          // [B][N][d]
  void *dqt, *dkt, *dvt;          // [B][m][d]: written when chunks == 1
  float* partial;                 // [B][chunks][3][m][d]: written when chunks > 1
  const int32_t* lens;            // valid history rows per user, nullable = all
  int N, m, d, chunks, chunk_rows;  // chunk_rows: history rows per chunk, a multiple of the workgroup's step
  float scale;
};
// waves per workgroup: two per SIMD where a wave fits 256 registers (d/h = 32, up to 64 links), one where it does not
constexpr int fused_waves(int dh, int link_blocks) { return dh == 32 && link_blocks <= 2 ? 8 : 4; }
template <int DH, int MB>
constexpr size_t fused_lds_bytes() {
  constexpr size_t copy = 3 * DH * 36 > 3 * 32 * 40 ? 3 * DH * 36 : 3 * 32 * 40, wave = 2 * (copy + 3 * 32 * 40), red = sizeof(float) * 3 * MB * (DH / 32) * 16 * 64;
  constexpr size_t links = 7 * MB * (DH / 16) * 64 * 16;  // seven fragment images of the links' operands
  return (fused_waves(DH, MB) * wave > red ? fused_waves(DH, MB) * wave : red) + links;
}
template <int DH, int MB>
__global__ __launch_bounds__(64 * fused_waves(DH, MB), 1) void xor_backward_fused_kernel(FusedArgs a) {
  constexpr int KS = DH / 16, TT = DH / 32;
  constexpr int kFusedWaves = fused_waves(DH, MB), kFusedStep = 32 * kFusedWaves;  // history rows per workgroup step
  // With up to two blocks of links the rows' sums wait until the last block is through (their accumulators do not fit
  // beside a block's tiles where two waves share a SIMD, nor beside the sums of 64 links at d/h = 64), each block's
  // tiles parked in a room of its own; with three or four blocks (d/h = 32, one wave per SIMD) each block's tiles go
  // into them right away, through one room.
  constexpr bool kDeferred = MB <= 2;
  constexpr int PITCH = 36;                 // transposed copy of a history tile: bf16 per row (8-byte reads, no bank conflicts)
  constexpr int P2 = DH + 8, CPR = DH / 8;  // staged rows: bf16 per row; 16-byte pieces per row
  constexpr int PP = 40;                    // parked p1, e1, e2: bf16 per history row (16-byte reads of 8 links)
  constexpr int kPark = 3 * 32 * PP, kCopy = 3 * DH * PITCH > kPark ? 3 * DH * PITCH : kPark;  // bf16 per wave: two rooms
  static_assert(kCopy >= kPark, "the last block's tiles are parked in the transposed copy's room");
  static_assert(kCopy >= 32 * P2, "and a staged block of rows fits it");
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, wv = tid / 64, lane = tid % 64, n = lane % 32, g = lane / 32, d = a.d;
  const int chunk = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int len = a.lens ? min(max(a.lens[b], 0), a.N) : a.N;
  const float inv_ns = len > 0 ? 1.f / static_cast<float>(len) : 0.f, inv_m = 1.f / static_cast<float>(a.m);
  const float minus_log2e_scale = -1.4426950408889634f * a.scale;
  // the factors left out of p1 = SiLU(s1) / n_S, e1 (scale / n_S) and p2, e2 (1 / m, scale / m), by accumulator:
  const float factor_s[3] = {a.scale * inv_ns, a.scale * inv_ns, a.scale * inv_m};  // dV[S] (p1), dK[S] (e1), dQ[S] (e2)
  const float factor_t[3] = {a.scale * inv_m, a.scale * inv_ns, a.scale * inv_m};   // dV[T] (p2), dQ[T] (e1), dK[T] (e2)
  bf16_any* yt = reinterpret_cast<bf16_any*>(smem) + wv * (kCopy + kPark);  // [3][DH][PITCH]: Q[S]^T, K[S]^T, G[S]^T
  bf16_any* pk = yt + kCopy;                                                // [3][32][PP]: p1, e1, e2 of one block
  bf16x8 zero;
#pragma unroll
  for (int t = 0; t < 8; ++t) zero[t] = static_cast<__bf16>(0.f);
  // A block of 32 links' rows (head slice), fetched row-contiguous (16 bytes per lane, DH/8 lanes per row) and staged
  // in the wave's piece of LDS; rows at or past m are read from row m - 1 instead and staged as zeros: the loads
  // themselves carry no condition.  (A uniform 64-bit base and a 32-bit offset per lane, here and below: addresses
  // take few registers; the host checks that a user's slab stays below 4 GiB.)
  auto stage_links = [&](const void* base, int lb) {
    const char* slab = static_cast<const char*>(base) + (static_cast<int64_t>(b) * a.m * d + head * DH) * 2;
    bf16x8 piece[KS];
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      const int idx = lane + 64 * i, row = min(32 * lb + idx / CPR, a.m - 1);
      piece[i] = *reinterpret_cast<const bf16x8*>(slab + static_cast<uint32_t>(row * d + 8 * (idx % CPR)) * 2u);
    }
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      const int idx = lane + 64 * i;
      *reinterpret_cast<bf16x8_any*>(yt + (idx / CPR) * P2 + 8 * (idx % CPR)) = 32 * lb + idx / CPR >= a.m ? zero : piece[i];
    }
  };
  // operand fragments of the staged block: lane (n, g) holds columns 16ks + 8g .. + 7 of row n
  auto fragments = [&](bf16x8 (&fr)[KS]) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fr[ks] = *reinterpret_cast<const bf16x8_any*>(yt + n * P2 + 16 * ks + 8 * g);
  };
  // and of its transpose: lane (n, g) holds rows 16kp + 8g .. + 7 of column 32tt + n
  auto transposed = [&](bf16x8 (&fr)[2][TT]) {
#pragma unroll
    for (int kp = 0; kp < 2; ++kp)
#pragma unroll
      for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int j = 0; j < 8; ++j) fr[kp][tt][j] = yt[(16 * kp + 8 * g + j) * P2 + 32 * tt + n];
  };
  const int c_begin = chunk * a.chunk_rows, c_end = min(c_begin + a.chunk_rows, a.N);
  // the wave's next tile of history rows: asked for one tile ahead
  struct Rows { bf16x8 q[KS], k[KS], v[KS], g[KS]; };
  Rows rows;
  const int c_stop = min(c_end, len);  // tiles from here on hold padding only
  // operand fragments straight from memory: lane (n, g) reads columns 16ks + 8g .. + 7 of row c0 + n (rows at or past
  // len from row len - 1 instead; they count as zeros when used)
  auto fetch_fragments = [&](const void* base, int c0, bf16x8 (&fr)[KS]) {
    if (base == nullptr) return;
    const char* slab = static_cast<const char*>(base) + (static_cast<int64_t>(b) * a.N * d + head * DH) * 2;
    const int row = min(c0 + n, len - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fr[ks] = *reinterpret_cast<const bf16x8*>(slab + static_cast<uint32_t>(row * d + 16 * ks + 8 * g) * 2u);
  };
  auto ask = [&](int c0) {
    if (c0 >= c_stop) return;
    fetch_fragments(a.qs, c0, rows.q), fetch_fragments(a.ks, c0, rows.k), fetch_fragments(a.vs, c0, rows.v), fetch_fragments(a.gs, c0, rows.g);
  };
  // (the first tile's rows are on their way while the links' operands are prepared)
  const int c_first = c_begin + 32 * wv;
  ask(c_first);
  // The links' operands, as fragment images in LDS shared by the waves (in registers they would not leave room
  // for the sums): B operands of the dot products (kinds 0-3: q, k, v, g; index ks) and transposed A operands of the
  // history rows' sums (kinds 4-6: q, k, g; index 2tt + kp).  Wave w prepares tensor w.
  constexpr int KF = DH / 16;
  bf16x8_any* links = reinterpret_cast<bf16x8_any*>(smem + fused_lds_bytes<DH, MB>() - 7 * MB * KF * 64 * 16);
  auto link_fragment = [&](int kind, int lb, int k) -> bf16x8_any& { return links[((kind * MB + lb) * KF + k) * 64 + lane]; };
  if (wv < 4) {
    const void* src = wv == 0 ? a.qt : (wv == 1 ? a.kt : (wv == 2 ? a.vt : a.gt));
#pragma unroll
    for (int lb = 0; lb < MB; ++lb) {
      bf16x8 fr[KS], tr[2][TT];
      stage_links(src, lb), fragments(fr);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) link_fragment(wv, lb, ks) = fr[ks];
      if (wv != 2) {
        transposed(tr);
#pragma unroll
        for (int kp = 0; kp < 2; ++kp)
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) link_fragment(wv == 3 ? 6 : 4 + wv, lb, 2 * tt + kp) = tr[kp][tt];
      }
    }
  }
  __syncthreads();
  f32x16 acc_t[3][MB][TT];  // dV[T]^T, dQ[T]^T, dK[T]^T: lane = link 32lb + n, register 4j + rr = head column 32tt + 8j + 4g + rr
#pragma unroll
  for (int o = 0; o < 3; ++o)
#pragma unroll
    for (int lb = 0; lb < MB; ++lb)
#pragma unroll
      for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc_t[o][lb][tt][i] = 0.f;
  // a tile's three gradients leave through the staged tile's room, so that a store instruction writes whole head
  // slices of a few rows (16 bytes per lane)
  bf16_t* outs[3] = {static_cast<bf16_t*>(a.dvs), static_cast<bf16_t*>(a.dks), static_cast<bf16_t*>(a.dqs)};
  auto store_rows = [&](bf16_t* out, int c0) {
#pragma unroll
    for (int i = 0; i < 32 * CPR / 64; ++i) {
      const int idx = lane + 64 * i, row = idx / CPR, piece = idx % CPR;
      const bf16x8 v = *reinterpret_cast<const bf16x8_any*>(yt + row * P2 + 8 * piece);
      char* slab = reinterpret_cast<char*>(out) + (static_cast<int64_t>(b) * a.N * d + head * DH) * 2;
      if (c0 + row < a.N) *reinterpret_cast<bf16x8_any*>(slab + static_cast<uint32_t>((c0 + row) * d + 8 * piece) * 2u) = v;
    }
  };
  for (int c0 = c_first; c0 < c_end; c0 += kFusedStep) {
    if (c0 >= len) {
      // padding only: zero gradients, nothing to read
#pragma unroll
      for (int i = 0; i < 32 * CPR / 64; ++i) *reinterpret_cast<bf16x8_any*>(yt + (lane + 64 * i) / CPR * P2 + 8 * ((lane + 64 * i) % CPR)) = zero;
#pragma unroll
      for (int o = 0; o < 3; ++o) store_rows(outs[o], c0);
      continue;
    }
    bf16x8 yq[KS], yk[KS], yv[KS], yg[KS];
    {
      const bool valid = c0 + n < len;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        yq[ks] = valid ? rows.q[ks] : zero, yk[ks] = valid ? rows.k[ks] : zero, yv[ks] = valid ? rows.v[ks] : zero;
        yg[ks] = (valid && a.gs != nullptr) ? rows.g[ks] : zero;
      }
    }
    // the transposed copy: column 16ks + 8g + t of row c0 + n goes to [column][n]
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int col = 16 * ks + 8 * g + t;
        yt[(0 * DH + col) * PITCH + n] = yq[ks][t];
        yt[(1 * DH + col) * PITCH + n] = yk[ks][t];
        yt[(2 * DH + col) * PITCH + n] = yg[ks][t];
      }
    // Per block of links: the two directions, the links' sums, and p1, e1, e2 parked for the rows' sums, which come
    // after the last block (their accumulators would not fit beside a block's tiles).  The last block's tiles are
    // parked in the transposed copy's room, which its links' sums are the last to read; the one before in a room of
    // its own.
    u16_any* park_room[2] = {reinterpret_cast<u16_any*>(pk), reinterpret_cast<u16_any*>(yt)};
    f32x16 acc_s[3][TT];  // dV[S]^T, dK[S]^T, dQ[S]^T: lane = row c0 + n, register 4j + rr = head column 32tt + 8j + 4g + rr
#pragma unroll
    for (int o = 0; o < 3; ++o)
#pragma unroll
      for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc_s[o][tt][i] = 0.f;
    // the rows' sums over one block's links, from its parked tiles
    auto rows_sums = [&](int lb, const u16_any* parked) {
      const bf16_any* room = reinterpret_cast<const bf16_any*>(parked);
#pragma unroll
      for (int kp = 0; kp < 2; ++kp) {
        const bf16x8 bp1 = *reinterpret_cast<const bf16x8_any*>(room + (0 * 32 + n) * PP + 16 * kp + 8 * g);
        const bf16x8 bf1 = *reinterpret_cast<const bf16x8_any*>(room + (1 * 32 + n) * PP + 16 * kp + 8 * g);
        const bf16x8 bf2 = *reinterpret_cast<const bf16x8_any*>(room + (2 * 32 + n) * PP + 16 * kp + 8 * g);
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
          acc_s[0][tt] = mfma32(link_fragment(6, lb, 2 * tt + kp), bp1, acc_s[0][tt]);  // dV[S]^T += G[T]^T p1^T
          acc_s[1][tt] = mfma32(link_fragment(4, lb, 2 * tt + kp), bf1, acc_s[1][tt]);  // dK[S]^T += Q[T]^T e1^T
          acc_s[2][tt] = mfma32(link_fragment(5, lb, 2 * tt + kp), bf2, acc_s[2][tt]);  // dQ[S]^T += K[T]^T e2^T
        }
        __builtin_amdgcn_sched_barrier(0);  // (a half's operands at a time)
      }
    };
#pragma unroll
    for (int lb = 0; lb < MB; ++lb) {
      // (the phases of a block are kept apart: moved into each other by the scheduler they need more registers than
      // two waves per SIMD leave)
      // Rounded to bf16 once, two registers to a word: a word's halves are what gets parked, four words are an
      // operand of the links' sums.  (The words are opaque to the compiler, which would otherwise convert again for
      // every 16-bit store.)
      unsigned wp1[8], we1[8], wp2[8], we2[8];
      auto round_pairs = [&](const f32x16& x, unsigned (&w)[8]) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          bf16x2 pair;
          pair[0] = static_cast<__bf16>(x[2 * k]), pair[1] = static_cast<__bf16>(x[2 * k + 1]);
          w[k] = __builtin_bit_cast(unsigned, pair);
          asm volatile("" : "+v"(w[k]));
        }
      };
      // One direction at a time: a logit tile z and a tile w of <G, V>, phi and phi' register by register up to the
      // constant factors, which the sums take at their end: z becomes SiLU(s) / scale, w becomes w SiLU'(s).
      auto direction = [&](const bf16x8 (&za)[KS], int zkind, const bf16x8 (&wa)[KS], int wkind, unsigned (&wp)[8], unsigned (&we)[8]) {
        __builtin_amdgcn_sched_barrier(0);
        f32x16 z, w;
#pragma unroll
        for (int i = 0; i < 16; ++i) z[i] = w[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          z = mfma32(za[ks], link_fragment(zkind, lb, ks), z);
          w = mfma32(wa[ks], link_fragment(wkind, lb, ks), w);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float gg = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(z[i] * minus_log2e_scale));
          z[i] *= gg;
          w[i] *= fmaf(z[i] * (1.f - gg), a.scale, gg);  // SiLU'(s) = g + s g (1 - g)
        }
        round_pairs(z, wp), round_pairs(w, we);
      };
      direction(yk, 0, yv, 3, wp1, we1);  // <K[S]_s, Q[T]_t>, <V[S]_s, G[T]_t>: p1, e1
      direction(yq, 1, yg, 2, wp2, we2);  // <Q[S]_s, K[T]_t>, <G[S]_s, V[T]_t>: p2, e2
      __builtin_amdgcn_sched_barrier(0);
      auto half_of = [&](const unsigned (&w)[8], int f) {
        u32x4 v;
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = w[4 * f + t];
        return __builtin_bit_cast(bf16x8, v);
      };
      // p1, e1, e2 parked as [history row][link]: registers 2k, 2k + 1 of lane (n, g) are rows 8 (k / 2) + 4g +
      // 2 (k % 2) and the next, link n
      auto park = [&](u16_any* room) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int row = 8 * (k / 2) + 4 * g + 2 * (k % 2);
          room[(0 * 32 + row) * PP + n] = static_cast<unsigned short>(wp1[k]), room[(0 * 32 + row + 1) * PP + n] = static_cast<unsigned short>(wp1[k] >> 16);
          room[(1 * 32 + row) * PP + n] = static_cast<unsigned short>(we1[k]), room[(1 * 32 + row + 1) * PP + n] = static_cast<unsigned short>(we1[k] >> 16);
          room[(2 * 32 + row) * PP + n] = static_cast<unsigned short>(we2[k]), room[(2 * 32 + row + 1) * PP + n] = static_cast<unsigned short>(we2[k] >> 16);
        }
      };
      if (kDeferred && lb < MB - 1) park(park_room[0]);
      __builtin_amdgcn_sched_barrier(0);
      // the links' sums over this tile's rows
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        const bf16x8 bp2 = half_of(wp2, f), be1 = half_of(we1, f), be2 = half_of(we2, f);
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
          // slot t of lane (n, g): row c0 + 16f + chain_k(g, t) of the history, head column 32tt + n
          auto chained = [&](int arr) {
            const bf16_any* src = yt + (arr * DH + 32 * tt + n) * PITCH + 16 * f + 4 * g;
            const bf16x4 lo = *reinterpret_cast<const bf16x4_any*>(src), hi = *reinterpret_cast<const bf16x4_any*>(src + 8);
            bf16x8 v;
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] = lo[t], v[4 + t] = hi[t];
            return v;
          };
          acc_t[0][lb][tt] = mfma32(chained(2), bp2, acc_t[0][lb][tt]);  // dV[T]^T += G[S]^T p2
          acc_t[1][lb][tt] = mfma32(chained(1), be1, acc_t[1][lb][tt]);  // dQ[T]^T += K[S]^T e1
          acc_t[2][lb][tt] = mfma32(chained(0), be2, acc_t[2][lb][tt]);  // dK[T]^T += Q[S]^T e2
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (kDeferred) {
        if (lb == MB - 1) park(park_room[1]);
      } else {
        park(park_room[0]);
        __builtin_amdgcn_sched_barrier(0);
        rows_sums(lb, park_room[0]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // (the next tile's rows are asked for here, every block's tiles and words used up: earlier there are no
    // registers for them, and the workgroup's other waves have work while this one waits for them)
    ask(c0 + kFusedStep);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (kDeferred) {
      // the rows' sums over all links
#pragma unroll
      for (int lb = 0; lb < MB; ++lb) rows_sums(lb, park_room[lb == MB - 1 ? 1 : 0]);
    }
#pragma unroll
    for (int o = 0; o < 3; ++o) {
#pragma unroll
      for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          bf16x4 v;
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) v[rr] = static_cast<__bf16>(acc_s[o][tt][4 * j + rr] * factor_s[o]);
          *reinterpret_cast<bf16x4_any*>(yt + n * P2 + 32 * tt + 8 * j + 4 * g) = v;
        }
      store_rows(outs[o], c0);
    }
  }
  // The waves' sums for the links meet in LDS, pairwise in a fixed order - (w, w + 4), then (w, w + 2), then (0, 1):
  // the upper half of the waves still in play writes, the lower half adds.  Four registers (four adjacent head
  // columns) to an LDS access.
  constexpr int kRed = 3 * MB * TT * 16 * 64;  // floats: one wave's accumulators
  static_assert(kFusedWaves / 2 * sizeof(float) * kRed <= fused_lds_bytes<DH, MB>(), "the slots fit the workgroup's LDS (all of it is free by now)");
  typedef float4 __attribute__((may_alias)) float4_any;
  float* red = reinterpret_cast<float*>(smem);
  auto slot_of = [&](int slot, int o, int lb, int tt, int j) {
    return reinterpret_cast<float4_any*>(red + slot * kRed) + (((o * MB + lb) * TT + tt) * 4 + j) * 64 + lane;
  };
  for (int half = kFusedWaves / 2; half >= 1; half /= 2) {
    __syncthreads();  // (the first one also ends every wave's use of its own piece and of the links' images; later ones the reads of a round)
    if (wv >= half && wv < 2 * half) {
#pragma unroll
      for (int o = 0; o < 3; ++o)
#pragma unroll
        for (int lb = 0; lb < MB; ++lb)
#pragma unroll
          for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const f32x16& x = acc_t[o][lb][tt];
              *slot_of(wv - half, o, lb, tt, j) = make_float4(x[4 * j], x[4 * j + 1], x[4 * j + 2], x[4 * j + 3]);
            }
    }
    __syncthreads();
    if (wv < half) {
#pragma unroll
      for (int o = 0; o < 3; ++o)
#pragma unroll
        for (int lb = 0; lb < MB; ++lb)
#pragma unroll
          for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const float4 y = *slot_of(wv, o, lb, tt, j);
              f32x16& x = acc_t[o][lb][tt];
              x[4 * j] += y.x, x[4 * j + 1] += y.y, x[4 * j + 2] += y.z, x[4 * j + 3] += y.w;
            }
    }
  }
  // Wave 0 holds the sums: laid out row-major in LDS ([output][link][head column], rows padded by four floats), so
  // that the workgroup stores whole head slices of a link's row, 16 bytes per lane.
  constexpr int RP = DH + 4;  // floats per row
  static_assert(3 * MB * 32 * RP <= kFusedWaves / 2 * kRed, "the row-major copy fits the slots");
  __syncthreads();
  if (wv == 0) {
#pragma unroll
    for (int o = 0; o < 3; ++o)
#pragma unroll
      for (int lb = 0; lb < MB; ++lb)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const f32x16& x = acc_t[o][lb][tt];
            // lane (n, g): link 32lb + n, head columns 32tt + 8j + 4g .. + 3
            *reinterpret_cast<float4_any*>(red + ((o * MB + lb) * 32 + n) * RP + 32 * tt + 8 * j + 4 * g) =
                make_float4(x[4 * j] * factor_t[o], x[4 * j + 1] * factor_t[o], x[4 * j + 2] * factor_t[o], x[4 * j + 3] * factor_t[o]);
          }
  }
  __syncthreads();
  const int64_t plane = static_cast<int64_t>(a.m) * d;
  constexpr int kQuads = 3 * MB * 32 * (DH / 4);  // 16-byte pieces of the three outputs
  for (int e = tid; e < kQuads; e += 64 * kFusedWaves) {
    const int quad = e % (DH / 4), row = (e / (DH / 4)) % (32 * MB), o = e / (DH / 4 * 32 * MB);
    if (row >= a.m) continue;
    const float4 v = *reinterpret_cast<const float4_any*>(red + (o * MB * 32 + row) * RP + 4 * quad);
    const int which = o == 0 ? 2 : (o == 1 ? 0 : 1);  // accumulators are (dV, dQ, dK); outputs are ordered (dQ, dK, dV)
    const int64_t at = (static_cast<int64_t>(b) * a.m + row) * d + head * DH + 4 * quad;
    if (a.chunks == 1) {
      bf16_t* out = static_cast<bf16_t*>(which == 0 ? a.dqt : (which == 1 ? a.dkt : a.dvt)) + at;
      store_as(out, v.x), store_as(out + 1, v.y), store_as(out + 2, v.z), store_as(out + 3, v.w);
    } else {
      *reinterpret_cast<float4*>(a.partial + ((static_cast<int64_t>(b) * a.chunks + chunk) * 3 + which) * plane +
                                 static_cast<int64_t>(row) * d + head * DH + 4 * quad) = v;
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

int step_rows(int dh, bool on_mfma) { return on_mfma ? kMfmaStep : (dh <= 32 ? 32 : 16); }

int chunks_for_links(int B, int N, int m, int h, int step) {
  // enough workgroups for two per compute unit, but no chunk shorter than one step
  const int64_t per_chunk = static_cast<int64_t>((m + kOwn - 1) / kOwn) * h * B;
  int64_t chunks = (2 * static_cast<int64_t>(compute_units()) + per_chunk - 1) / per_chunk;
  const int64_t steps = (N + step - 1) / step;
  if (chunks > steps) chunks = steps;
  if (chunks < 1) chunks = 1;
  return static_cast<int>(chunks);
}

template <typename T>
hipError_t launch_side(const SideArgs& a, dim3 grid, bool on_mfma, bool own_per_wave, hipStream_t s) {
  if (on_mfma && a.dh == 32 && own_per_wave)
    hipLaunchKernelGGL((xor_backward_side_mfma_kernel<32, true>), grid, dim3(256), 0, s, a);
  else if (on_mfma && a.dh == 32)
    hipLaunchKernelGGL((xor_backward_side_mfma_kernel<32, false>), grid, dim3(256), 0, s, a);
  else if (on_mfma && own_per_wave)
    hipLaunchKernelGGL((xor_backward_side_mfma_kernel<64, true>), grid, dim3(256), 0, s, a);
  else if (on_mfma)
    hipLaunchKernelGGL((xor_backward_side_mfma_kernel<64, false>), grid, dim3(256), 0, s, a);
  else if (a.dh <= 32)
    hipLaunchKernelGGL((xor_backward_side_kernel<T, 32, 32>), grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((xor_backward_side_kernel<T, kMaxDh, 16>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The one-pass form: at most 128 links at d/h = 32, 64 at d/h = 64 (the links' sums must fit a wave's registers).
constexpr int kFusedLinks32 = 128, kFusedLinks64 = 64;  // by head width
bool fused_shape(int N, int m, int d, int dh) {
  return ((dh == 32 && m <= kFusedLinks32) || (dh == 64 && m <= kFusedLinks64)) &&
         static_cast<int64_t>(N) * d * 2 < (int64_t{1} << 32);  // (32-bit offsets within a user)
}
int chunks_for_fused(int B, int N, int h, int dh, int m) {
  const int kFusedStep = 32 * fused_waves(dh, (m + 31) / 32);
  // one workgroup per compute unit (a wave per SIMD), but no chunk shorter than one step
  const int64_t per_chunk = static_cast<int64_t>(h) * B;
  const int64_t steps = (N + kFusedStep - 1) / kFusedStep;
  int64_t chunks = std::min<int64_t>(steps, (compute_units() + per_chunk - 1) / per_chunk);
  if (chunks < 1) chunks = 1;
  const int64_t steps_per_chunk = (steps + chunks - 1) / chunks;
  return static_cast<int>((steps + steps_per_chunk - 1) / steps_per_chunk);  // no empty chunk
}

template <int DH, int MB>
hipError_t launch_fused(const FusedArgs& a, dim3 grid, hipStream_t s) {
  auto kernel = xor_backward_fused_kernel<DH, MB>;
  constexpr size_t lds = fused_lds_bytes<DH, MB>();
  static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kernel, grid, dim3(64 * fused_waves(DH, MB)), lds, s, a);
  return hipGetLastError();
}

hipError_t xor_backward_fused(const XorBackward& g, void* workspace, hipStream_t s) {
  FusedArgs a{};
  a.qs = g.QS, a.ks = g.KS, a.vs = g.VS, a.gs = g.dOS, a.qt = g.QT, a.kt = g.KT, a.vt = g.VT, a.gt = g.dOT;
  a.dqs = g.dQS, a.dks = g.dKS, a.dvs = g.dVS, a.dqt = g.dQT, a.dkt = g.dKT, a.dvt = g.dVT;
  a.partial = static_cast<float*>(workspace), a.lens = g.lens;
  a.N = g.N, a.m = g.m, a.d = g.d, a.scale = g.scale;
  const int dh = g.d / g.h, blocks = (g.m + 31) / 32, kFusedStep = 32 * fused_waves(dh, blocks);
  a.chunks = chunks_for_fused(g.B, g.N, g.h, dh, g.m);
  const int steps = (g.N + kFusedStep - 1) / kFusedStep;
  a.chunk_rows = (steps + a.chunks - 1) / a.chunks * kFusedStep;
  const dim3 grid(a.chunks, g.h, g.B);
  hipError_t e = hipErrorInvalidValue;
  if (dh == 32) {
    e = blocks == 1 ? launch_fused<32, 1>(a, grid, s) : blocks == 2 ? launch_fused<32, 2>(a, grid, s)
      : blocks == 3 ? launch_fused<32, 3>(a, grid, s) : launch_fused<32, 4>(a, grid, s);
  } else {
    e = blocks == 1 ? launch_fused<64, 1>(a, grid, s) : launch_fused<64, 2>(a, grid, s);
  }
  if (e != hipSuccess || a.chunks == 1) return e;
  const int64_t plane = static_cast<int64_t>(g.m) * g.d;
  hipLaunchKernelGGL(xor_backward_reduce_kernel<bf16_t>, dim3(static_cast<unsigned>((plane + 255) / 256), 3, g.B), dim3(256), 0, s,
                     static_cast<const float*>(workspace), static_cast<bf16_t*>(g.dQT), static_cast<bf16_t*>(g.dKT),
                     static_cast<bf16_t*>(g.dVT), a.chunks, plane);
  return hipGetLastError();
}

template <typename T>
hipError_t xor_backward_typed(const XorBackward& g, void* workspace, hipStream_t s) {
  SideArgs a{};
  a.lens = g.lens, a.d = g.d, a.dh = g.d / g.h, a.scale = g.scale;
  // the matrix-core form reads 16-byte pieces of bf16 rows
  bool on_mfma = g.dtype == 1 && (a.dh == 32 || a.dh == 64);
  for (const void* p : {g.QS, g.KS, g.VS, g.QT, g.KT, g.VT, g.dOT, g.dOS}) on_mfma = on_mfma && aligned16(p);
  for (const void* p : {g.dQS, g.dKS, g.dVS}) on_mfma = on_mfma && aligned16(p);  // (stored 16 bytes at a time)
  if (on_mfma && fused_shape(g.N, g.m, g.d, a.dh)) return xor_backward_fused(g, workspace, s);
  const int step = step_rows(a.dh, on_mfma);
  // history side: every block of 32 history rows against all links
  a.qx = g.QS, a.kx = g.KS, a.vx = g.VS, a.gx = g.dOS;
  a.qy = g.QT, a.ky = g.KT, a.vy = g.VT, a.gy = g.dOT;
  a.dq = g.dQS, a.dk = g.dKS, a.dv = g.dVS, a.partial = nullptr;
  a.own_is_history = 1, a.rows_x = g.N, a.rows_y = g.m, a.chunks = 1;
  a.chunk_rows = (g.m + step - 1) / step * step;
  // (on the matrix cores a workgroup takes 128 history rows, one wave per 32, each wave against all links)
  const int own_rows = on_mfma ? 4 * kOwn : kOwn;
  hipError_t e = launch_side<T>(a, dim3((g.N + own_rows - 1) / own_rows, g.h, g.B), on_mfma, true, s);
  if (e != hipSuccess) return e;
  // link side: every block of 32 links against the history rows, in chunks
  const int chunks = chunks_for_links(g.B, g.N, g.m, g.h, step);
  a.qx = g.QT, a.kx = g.KT, a.vx = g.VT, a.gx = g.dOT;
  a.qy = g.QS, a.ky = g.KS, a.vy = g.VS, a.gy = g.dOS;
  a.dq = g.dQT, a.dk = g.dKT, a.dv = g.dVT, a.partial = static_cast<float*>(workspace);
  a.own_is_history = 0, a.rows_x = g.m, a.rows_y = g.N, a.chunks = chunks;
  const int steps = (g.N + step - 1) / step;
  a.chunk_rows = (steps + chunks - 1) / chunks * step;
  const int blocks_x = (g.m + kOwn - 1) / kOwn;
  e = launch_side<T>(a, dim3(blocks_x * chunks, g.h, g.B), on_mfma, false, s);
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
  // large enough for either kernel (a bf16 call whose pointers are not 16-byte aligned runs on the vector ALUs)
  int chunks = std::max(chunks_for_links(B, N, m, h, step_rows(d / h, false)),
                        chunks_for_links(B, N, m, h, step_rows(d / h, true)));
  if (fused_shape(N, m, d, d / h)) chunks = std::max(chunks, chunks_for_fused(B, N, h, d / h, m));
  return chunks == 1 ? 256 : align_up(static_cast<size_t>(B) * chunks * 3 * m * d * sizeof(float));
}

hipError_t xor_backward(const XorBackward& g, void* workspace, hipStream_t s) {
  return g.dtype == 0 ? xor_backward_typed<float>(g, workspace, s) : xor_backward_typed<bf16_t>(g, workspace, s);
}

}  // namespace lime
