// Operand packing for the matrix-core kernels: weight matrices and the small projected link
// matrices (m rows) are written once per call in MFMA fragment order.
#include "mfma.hpp"

namespace lime {
namespace {

constexpr int kPackRows = 4;   // rows of X per block of a projection job
constexpr int kPackCols = 32;  // columns of W per block
constexpr int kMaxJobs = kMaxPackProjections, kMaxWeights = kMaxPackWeights;

struct PackArgs {
  const bf16_t* w_src[kMaxWeights];
  bf16x8* w_img[kMaxWeights];
  float w_sign[kMaxWeights];
  int w_pad[kMaxWeights];
  const bf16_t* p_x[kMaxJobs];
  const bf16_t* p_w[kMaxJobs];
  bf16_t* p_img[kMaxJobs];
  int64_t p_stride[kMaxJobs];
  int p_layout[kMaxJobs];
  float p_sign[kMaxJobs];
  const bf16_t* p_gamma[kMaxJobs];  // layer normalisation of a job's rows before its projection (p_norm set)
  const bf16_t* p_beta[kMaxJobs];
  float p_eps[kMaxJobs];
  int p_norm[kMaxJobs];
  int p_first_block[kMaxJobs + 1];  // block ranges of the projection jobs, after the weight jobs
  const bf16_t *s_wq, *s_k, *s_wk;  // the score job (at most one), after the projection jobs
  bf16_t* s_img;
  float s_sign;
  int n_weights, blocks_per_weight;
  int d, dh, m;
};

// One wavefront of a score job: the 32 x 32 block (links 32lb.., rows j = 32jb..) of head a's
//   G_a^T[l][j] = sum_c K~[l][a dh + c] Wq[j][a dh + c],   K~ = Ksrc Wk,
// computed on the matrix cores as Ksrc (Wk_a Wq_a^T): in that order both products read their operands row-major
// with the summed index contiguous, so no transposed copy of a weight is needed.  For each block of 32 rows k of
// Wk the wave forms M = Wk_a[k-block] Wq_a[j-block]^T (summed over the head's columns) and feeds it straight back
// as the B operand of Ksrc[l-block][k-block] . M (chained order, see mfma.hpp).
template <int DH, int M, int NKB>
__device__ void score_wave(const PackArgs& p, int combo) {
  constexpr int D = 32 * NKB, H = D / DH, LB = M / 32, KC = DH / 16, K1 = D / 16;
  const int lane = threadIdx.x & 63, n = lane & 31, g = lane >> 5;
  const int lb = combo % LB, jb = (combo / LB) % NKB, a = combo / (LB * NKB);
  if (a >= H) return;  // uniform over the wave
  // a null weight stands for the identity
  auto rows_of = [&](const bf16_t* W, int row, int kc) {
    const int c0 = a * DH + 16 * kc + 8 * g;
    if (W != nullptr) return *reinterpret_cast<const bf16x8*>(W + static_cast<int64_t>(row) * D + c0);
    bf16x8 v;
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = static_cast<__bf16>(row == c0 + t ? 1.f : 0.f);
    return v;
  };
  bf16x8 wq[KC], wk[NKB][KC], lf[NKB][2];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) wq[kc] = rows_of(p.s_wq, 32 * jb + n, kc);
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) wk[kb][kc] = rows_of(p.s_wk, 32 * kb + n, kc);
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      // slot t stands for k = 32kb + 16f + chain_k(g, t): columns 4g..4g+3 and 8+4g..8+4g+3 of the 16
      const bf16_t* src = p.s_k + static_cast<int64_t>(32 * lb + n) * D + 32 * kb + 16 * f + 4 * g;
      const bf16x4 lo = *reinterpret_cast<const bf16x4*>(src), hi = *reinterpret_cast<const bf16x4*>(src + 8);
#pragma unroll
      for (int t = 0; t < 4; ++t) lf[kb][f][t] = lo[t], lf[kb][f][4 + t] = hi[t];
    }
  }
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    f32x16 mk;
#pragma unroll
    for (int i = 0; i < 16; ++i) mk[i] = 0.f;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) mk = mfma32(wk[kb][kc], wq[kc], mk);
#pragma unroll
    for (int f = 0; f < 2; ++f) acc = mfma32(lf[kb][f], pack_half(mk, f), acc);
  }
  // register 4jj + r is link 32lb + 8jj + 4g + r, the lane's column is row j = 32jb + n of G_a
  const int j = 32 * jb + n;
  const int64_t frag = (static_cast<int64_t>(a) * K1 + j / 16) * LB + lb + a * kQueryImageHeadPad;
  bf16_t* dst = p.s_img + (frag * 64 + 32 * ((j % 16) / 8)) * 8 + j % 8;
#pragma unroll
  for (int i = 0; i < 16; ++i) store_as(dst + (8 * (i / 4) + 4 * g + i % 4) * 8, acc[i] * p.s_sign);
}

// SDH, SM, SNKB: shape of the score job (d/h, m, d/32) this instance can run after its other jobs; 0 = none.
template <int SDH, int SM, int SNKB>
__global__ __launch_bounds__(256) void pack_kernel(PackArgs p) {
  extern __shared__ float smem[];
  const int d = p.d, dh = p.dh, m = p.m, tid = threadIdx.x;
  int blk = blockIdx.x;
  if constexpr (SDH != 0) {
    if (blk >= p.n_weights * p.blocks_per_weight + p.p_first_block[kMaxJobs]) {  // uniform
      blk -= p.n_weights * p.blocks_per_weight + p.p_first_block[kMaxJobs];
      score_wave<SDH, SM, SNKB>(p, blk * 4 + tid / 64);
      return;
    }
  }
  if (blk < p.n_weights * p.blocks_per_weight) {
    // one thread per (8 consecutive k, column): a 16-byte slot of the weight image
    const int job = blk / p.blocks_per_weight;
    const int idx = (blk % p.blocks_per_weight) * 256 + tid;
    if (idx >= d * d / 8) return;
    const bf16_t* W = p.w_src[job];
    const int col = idx % d, k0 = (idx / d) * 8;
    // (one uniform branch around all eight loads: a test per element would make each load wait for the one before)
    float x[8];
    if (W != nullptr) {
      bf16_t raw[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) raw[t] = W[static_cast<int64_t>(k0 + t) * d + col];
#pragma unroll
      for (int t = 0; t < 8; ++t) x[t] = to_float(raw[t]);
    } else {
#pragma unroll
      for (int t = 0; t < 8; ++t) x[t] = k0 + t == col ? 1.f : 0.f;
    }
    bf16x8 v;
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = static_cast<__bf16>(x[t] * p.w_sign[job]);
    const int a = col / dh, c = col % dh, mb = c / 32, n = c % 32;
    const int kk = k0 / 16, g = (k0 % 16) / 8;
    const int64_t frag = (static_cast<int64_t>(a) * (d / 16) + kk) * (dh / 32) + mb;
    p.w_img[job][(frag + a * p.w_pad[job]) * 64 + 32 * g + n] = v;
    return;
  }
  blk -= p.n_weights * p.blocks_per_weight;
  const int job = blk >= p.p_first_block[2] ? 2 : (blk >= p.p_first_block[1] ? 1 : 0);
  blk -= p.p_first_block[job];
  // A block computes kPackRows rows x kPackCols columns of X W: it fetches only its column slice of W
  // (d x kPackCols), so that no compute unit has to take in the whole matrix.  Thread (cg, kc) owns 8
  // adjacent columns and every nkc-th k; the partial sums meet in LDS.
  const int slices = d / kPackCols, groups = m / kPackRows;  // d is a multiple of 32, m of 32
  const int slice = blk % slices, rg = (blk / slices) % groups, u = blk / (slices * groups);
  const int row0 = rg * kPackRows, col0 = slice * kPackCols;
  const bf16_t* X = p.p_x[job] + u * p.p_stride[job] + static_cast<int64_t>(row0) * d;
  const bf16_t* W = p.p_w[job];

  float* xs = smem;                          // [kPackRows][d]
  float* out = xs + kPackRows * d;           // [kPackRows][kPackCols]
  float* red = out + kPackRows * kPackCols;  // [nkc][kPackRows * kPackCols + 1]: the odd pitch spreads the k-groups over the banks
  constexpr int CG = kPackCols / 8, nkc = 256 / CG;
  constexpr int kMaxK = 256 / nkc;  // k-steps per thread at the largest d (256)
  constexpr int kRedPitch = kPackRows * kPackCols + 1;
  const int cg = tid % CG, kc = tid / CG;
  // every load this block needs is issued before the first wait
  bf16x8 wreg[kMaxK];
  if (W != nullptr) {
#pragma unroll
    for (int it = 0; it < kMaxK; ++it) {
      const int k = kc + it * nkc;
      if (k < d) wreg[it] = *reinterpret_cast<const bf16x8*>(W + static_cast<int64_t>(k) * d + col0 + 8 * cg);
    }
  }
  // (scale and shift of a normalised job: asked for with everything else, used after the rows have arrived; a lane
  // takes pairs of neighbouring columns so that they come as 32-bit loads, which nothing touches before their use)
  constexpr int kNormPairs = 256 / 128;  // column pairs per lane at the largest d
  uint32_t ln_g[kNormPairs], ln_b[kNormPairs];
  if (p.p_norm[job]) {
#pragma unroll
    for (int i = 0; i < kNormPairs; ++i) {
      const int k = min(2 * (tid % 64) + 128 * i, d - 2);
      ln_g[i] = reinterpret_cast<const uint32_t*>(p.p_gamma[job])[k / 2];
      ln_b[i] = reinterpret_cast<const uint32_t*>(p.p_beta[job])[k / 2];
    }
  }
  for (int i = tid; i < kPackRows * d; i += 256) xs[i] = to_float(X[i]);
  __syncthreads();
  if (p.p_norm[job]) {
    // one wavefront per row (kPackRows of them): mean, centred second moment, then the normalised row rounded to
    // bf16, as a normalisation pass of its own would have stored it
    static_assert(kPackRows * 64 == 256, "a wavefront per row");
    float* xr = xs + (tid / 64) * d;
    float x[2 * kNormPairs], sum = 0.f;
#pragma unroll
    for (int i = 0; i < kNormPairs; ++i) {
      const int k = 2 * (tid % 64) + 128 * i;
      x[2 * i] = k < d ? xr[k] : 0.f, x[2 * i + 1] = k < d ? xr[k + 1] : 0.f;
      sum += x[2 * i] + x[2 * i + 1];
    }
    const float mean = wave_sum(sum) / static_cast<float>(d);
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < kNormPairs; ++i) {
      const int k = 2 * (tid % 64) + 128 * i;
      x[2 * i] = k < d ? x[2 * i] - mean : 0.f, x[2 * i + 1] = k < d ? x[2 * i + 1] - mean : 0.f;
      q = fmaf(x[2 * i], x[2 * i], fmaf(x[2 * i + 1], x[2 * i + 1], q));
    }
    const float inv = 1.f / sqrtf(wave_sum(q) / static_cast<float>(d) + p.p_eps[job]);
#pragma unroll
    for (int i = 0; i < kNormPairs; ++i) {
      const int k = 2 * (tid % 64) + 128 * i;
      if (k < d) {
        xr[k] = static_cast<float>(static_cast<__bf16>(
            fmaf(x[2 * i] * inv, __uint_as_float(ln_g[i] << 16), __uint_as_float(ln_b[i] << 16))));
        xr[k + 1] = static_cast<float>(static_cast<__bf16>(
            fmaf(x[2 * i + 1] * inv, __uint_as_float(ln_g[i] & 0xffff0000u), __uint_as_float(ln_b[i] & 0xffff0000u))));
      }
    }
    __syncthreads();
  }
  if (W == nullptr) {
    for (int i = tid; i < kPackRows * kPackCols; i += 256) out[i] = xs[(i / kPackCols) * d + col0 + i % kPackCols];
  } else {
    float acc[kPackRows][8];
#pragma unroll
    for (int r = 0; r < kPackRows; ++r)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[r][j] = 0.f;
#pragma unroll
    for (int it = 0; it < kMaxK; ++it) {
      const int k = kc + it * nkc;
      if (k < d) {
#pragma unroll
        for (int r = 0; r < kPackRows; ++r) {
          const float x = xs[r * d + k];
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[r][j] = fmaf(x, static_cast<float>(wreg[it][j]), acc[r][j]);
        }
      }
    }
#pragma unroll
    for (int r = 0; r < kPackRows; ++r)
#pragma unroll
      for (int j = 0; j < 8; ++j) red[kc * kRedPitch + r * kPackCols + 8 * cg + j] = acc[r][j];
    __syncthreads();
    for (int i = tid; i < kPackRows * kPackCols; i += 256) {
      float sum = 0.f;
#pragma unroll 8
      for (int c = 0; c < nkc; ++c) sum += red[c * kRedPitch + i];
      out[i] = sum;
    }
  }
  __syncthreads();
  bf16_t* img = p.p_img[job];
  const bool keys = p.p_layout[job] == kPackKeys;
  const float sign = p.p_sign[job];
  for (int i = tid; i < kPackRows * kPackCols; i += 256) {
    const int row = row0 + i / kPackCols, col = col0 + i % kPackCols;
    store_as(img + (keys ? keys_slot(u, row, col, d, dh, m) : values_slot(u, row, col, d, dh, m, p.p_layout[job] == kPackValues)), sign * out[i]);
  }
}

}  // namespace

hipError_t pack_operands(const PackWeight* weights, int n_weights, const PackProject* projections, int n_projections,
                         int d, int h, int m, hipStream_t s, const PackScore* score) {
  if (n_weights > kMaxWeights || n_projections > kMaxJobs) return hipErrorInvalidValue;
  PackArgs p{};
  p.d = d, p.dh = d / h, p.m = m;
  p.n_weights = n_weights;
  p.blocks_per_weight = (d * d / 8 + 255) / 256;
  for (int i = 0; i < n_weights; ++i) {
    p.w_src[i] = static_cast<const bf16_t*>(weights[i].W);
    p.w_img[i] = static_cast<bf16x8*>(weights[i].image);
    p.w_sign[i] = weights[i].sign;
    p.w_pad[i] = weights[i].head_pad;
  }
  int blocks = 0;
  for (int i = 0; i < kMaxJobs; ++i) {
    p.p_first_block[i] = blocks;
    if (i < n_projections) {
      p.p_x[i] = static_cast<const bf16_t*>(projections[i].X);
      p.p_w[i] = static_cast<const bf16_t*>(projections[i].W);
      p.p_img[i] = static_cast<bf16_t*>(projections[i].image);
      p.p_stride[i] = projections[i].user_stride;
      p.p_layout[i] = projections[i].layout;
      p.p_sign[i] = projections[i].sign;
      p.p_norm[i] = projections[i].norm.on ? 1 : 0;
      p.p_gamma[i] = static_cast<const bf16_t*>(projections[i].norm.gamma);
      p.p_beta[i] = static_cast<const bf16_t*>(projections[i].norm.beta);
      p.p_eps[i] = projections[i].norm.eps;
      blocks += projections[i].users * (m / kPackRows) * (d / kPackCols);
    }
  }
  p.p_first_block[kMaxJobs] = blocks;
  for (int i = n_projections; i < kMaxJobs; ++i)
    if (i > 0) p.p_first_block[i] = 0x7fffffff;
  constexpr int nkc = 256 / (kPackCols / 8);
  size_t lds = (static_cast<size_t>(kPackRows) * d + static_cast<size_t>(1 + nkc) * kPackRows * kPackCols + nkc) * sizeof(float);
  int grid = n_weights * p.blocks_per_weight + blocks;
  if (score == nullptr) {
    if (grid == 0) return hipSuccess;
    hipLaunchKernelGGL((pack_kernel<0, 0, 0>), dim3(grid), dim3(256), lds, s, p);
    return hipGetLastError();
  }
  p.s_wq = static_cast<const bf16_t*>(score->Wq), p.s_k = static_cast<const bf16_t*>(score->Ksrc);
  p.s_wk = static_cast<const bf16_t*>(score->Wk), p.s_img = static_cast<bf16_t*>(score->image);
  p.s_sign = score->sign;
  const int dh = d / h, nkb = d / 32;
  grid += (h * nkb * (m / 32) + 3) / 4;  // four wavefronts per block, one 32 x 32 block of the image each
#define LIME_SCORE_CASE(DH_, M_, NKB_)                                                              \
  if (dh == DH_ && m == M_ && nkb == NKB_) {                                                        \
    hipLaunchKernelGGL((pack_kernel<DH_, M_, NKB_>), dim3(grid), dim3(256), lds, s, p);             \
    return hipGetLastError();                                                                       \
  }
  LIME_SCORE_CASE(64, 64, 8) LIME_SCORE_CASE(64, 64, 4) LIME_SCORE_CASE(64, 64, 2)
  LIME_SCORE_CASE(64, 32, 8) LIME_SCORE_CASE(64, 32, 4) LIME_SCORE_CASE(64, 32, 2)
  LIME_SCORE_CASE(32, 32, 8) LIME_SCORE_CASE(32, 32, 4) LIME_SCORE_CASE(32, 32, 2) LIME_SCORE_CASE(32, 32, 1)
#undef LIME_SCORE_CASE
  return hipErrorInvalidValue;
}

hipError_t pack_operands(const PackJobs& jobs, int d, int h, int m, hipStream_t s) {
  return pack_operands(jobs.weights, jobs.n_weights, jobs.projections, jobs.n_projections, d, h, m, s,
                       jobs.has_score ? &jobs.score : nullptr);
}

PreparedLayout prepared_layout(int d, int m) {
  PreparedLayout l{};
  const size_t w = align_up(static_cast<size_t>(d) * d * 2 + kQueryImagePadBytes), links = align_up(static_cast<size_t>(m) * d * 2);
  l.wk = 0, l.wv = w, l.qb = 2 * w, l.wq = 2 * w + links, l.ka = 3 * w + links, l.total = 3 * w + 2 * links;
  return l;
}

hipError_t prepare_operands(const PrepareOperands& p, void* prepared, hipStream_t s) {
  const PreparedLayout l = prepared_layout(p.d, p.m);
  char* base = static_cast<char*>(prepared);
  const float sign_cand = p.scale_cand < 0.f ? -1.f : 1.f;
  PackWeight wjobs[3] = {{p.Wk_hist, base + l.wk}, {p.Wv_hist, base + l.wv}, {p.Wq_cand, base + l.wq, 1.f, kQueryImageHeadPad}};
  PackProject pjobs[2] = {{p.LC, p.Wq_hist, base + l.qb, 0, 1, kPackKeys, p.scale_hist < 0.f ? -1.f : 1.f},
                          {p.L, p.Wk_cand, base + l.ka, 0, 1, kPackKeys, sign_cand}};
  if (fused_scores(p.d, p.h, p.m, false)) {
    // the candidate stage then wants G = W_Q (L W_K)^T per head in place of W_Q^T and K~
    PackScore sjob{p.Wq_cand, p.L, p.Wk_cand, base + l.wq, sign_cand};
    return pack_operands(wjobs, 2, pjobs, 1, p.d, p.h, p.m, s, &sjob);
  }
  return pack_operands(wjobs, 3, pjobs, 2, p.d, p.h, p.m, s);
}

}  // namespace lime
