// User-side link personalisation on the matrix cores: the m links attend over the N history
// rows, by softmax (Eq. 3) or by the target-to-source half of XORA, O[T] (Eq. 7, phi = SiLU/n_s).
//
// Design: one fused pass over E.  A workgroup is a single wavefront that owns one head of a chunk
// of one user's history (histories are short next to the chip: many small workgroups keep every
// compute unit busy and each fetches only its own head's operands).  The wave keeps the head's
// slices of W_K^T and W_V and the projected link queries Q~_a in fragment form (W_K^T in LDS when
// d = 256, otherwise in registers) and walks its chunk in tiles of 32 items, requesting the next
// tile's rows before it computes the current one.  Per tile, with X = the 32 history rows read
// row-major as stored:
//   K~^T (d/h x 32) = W_K,a^T . X^T     X is the B operand
//   V~   (32 x d/h) = X . W_V,a         the same X registers are the A operand
//   S^T  (32 x m)   = K~ . Q~_a^T       A operand = accumulators of the first product
//   L^P^T(d/h x m) += V~^T . phi(S)^T   both operands are accumulators (of the 2nd and 3rd product)
// so the projected keys and values never leave registers.  Each lane owns one link (column of
// S^T and of L^P^T): the running softmax maximum, the running sum and the rescaling of the
// accumulator are all lane-local, plus one exchange with lane ^ 32.  Rows at or beyond lens[b] are
// replaced by zeros as they are loaded and masked out of phi, so their content is never used.
// Every chunk writes an un-normalised partial (max, sum, accumulator); a small merge kernel
// combines the chunks of a user in a fixed order (deterministic) and writes L^P.
#include "mfma.hpp"

namespace lime {
namespace {

constexpr float kLog2e = 1.4426950408889634f;

struct HistArgs {
  const bf16_t* E;
  const int32_t* lens;
  const bf16x8 *WkA, *WvB, *QB;
  int64_t qb_user_frags;  // size of one user's query image in bf16x8 units (0 = shared links)
  float* part_acc;        // [B][chunks][h][m][dh]
  float* part_ml;         // [B][chunks][h][m][2]  (running max, running sum)
  int N, chunk_items, chunks;
  float scale;
};

// COOP = false: a workgroup is one wave (one head of one chunk; grid.z = heads) that reads its rows
// straight from memory, one tile ahead.  COOP = true (long histories, d <= 128): a workgroup is h waves
// (all heads of one chunk) that copy each tile once, cooperatively and several tiles ahead, through a
// register ring into LDS, as the candidate-side kernel does.
template <int DH, int M, int H, int PHI, bool WK_LDS, bool COOP>
__global__ __launch_bounds__(COOP ? 64 * H : 64) void links_over_history_kernel(HistArgs a) {
  constexpr int D = DH * H;
  constexpr int K1 = D / 16, MB = DH / 32;  // projections: k-steps over d, blocks over d/h
  constexpr int K2 = DH / 16, LB = M / 32;  // scores: k-steps over d/h, blocks over links
  constexpr int P = WK_LDS ? (M >= 128 ? 1 : 2) : 4;  // COOP: tiles in flight per workgroup (registers permitting)
  constexpr int NXS = COOP ? (WK_LDS ? 1 : 2) : 1;  // COOP: LDS tile buffers (one when W_K^T fills the LDS)
  constexpr int LW = DH / 16;               // COOP: 1 KiB loads per wave and tile
  constexpr int CPR = D / 8, PITCH = 2 * D + 16;
  extern __shared__ bf16x8 lds_wk_all[];
  __shared__ __attribute__((aligned(16))) unsigned char xs[NXS][COOP ? 32 * PITCH : 16];
  const int lane = threadIdx.x & 63, head = COOP ? threadIdx.x >> 6 : blockIdx.z;
  const int n = lane & 31, g = lane >> 5;
  const int b = blockIdx.y, chunk = blockIdx.x;
  const int len = a.lens ? min(a.lens[b], a.N) : a.N;
  const int i_begin = chunk * a.chunk_items;
  if (i_begin >= len) return;  // uniform over the workgroup: nothing for this chunk
  const int i_end = min(len, i_begin + a.chunk_items);

  const bf16_t* Eb = a.E + static_cast<int64_t>(b) * a.N * D;
  // rows at or beyond the end of the chunk are replaced by zeros (their content is never used)
  auto load_tile = [&](int i0, bf16x8 (&x)[K1]) {
    const int item = i0 + n;
    const bf16_t* xrow = Eb + static_cast<int64_t>(min(item, a.N - 1)) * D + 8 * g;
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) {
      bf16x8 v;
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = static_cast<__bf16>(0.f);
      if (item < i_end) v = *reinterpret_cast<const bf16x8*>(xrow + 16 * kk);
      x[kk] = v;
    }
  };
  // The first tile's rows come from HBM and are asked for ahead of the operands, which come from L2: behind them, as
  // the loop's own order has it, their latency would begin only once the operands had arrived (the W_K^T slice is
  // waited for on its way into LDS).
  bf16x8 xnext[COOP ? 1 : K1];
  if constexpr (!COOP) load_tile(i_begin, xnext);

  bf16x8* lds_wk = lds_wk_all + (COOP ? head * K1 * MB * 64 : 0);  // this wave's slice
  bf16x8 wk[WK_LDS ? 1 : K1][WK_LDS ? 1 : MB];
  if (WK_LDS) {
    // this head's W_K^T image: the lane moves exactly the K1*MB fragments it will read back itself
    bf16x8 tmp[K1 * MB];
#pragma unroll
    for (int it = 0; it < K1 * MB; ++it) tmp[it] = a.WkA[(head * K1 * MB + it) * 64 + lane];
#pragma unroll
    for (int it = 0; it < K1 * MB; ++it) lds_wk[it * 64 + lane] = tmp[it];
  } else {
#pragma unroll
    for (int kk = 0; kk < K1; ++kk)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) wk[kk][mb] = a.WkA[((head * K1 + kk) * MB + mb) * 64 + lane];
  }
  bf16x8 wv[K1][MB];
#pragma unroll
  for (int kk = 0; kk < K1; ++kk)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) wv[kk][mb] = a.WvB[((head * K1 + kk) * MB + mb) * 64 + lane];
  bf16x8 qb[K2][LB];
  {
    const bf16x8* src = a.QB + b * a.qb_user_frags + static_cast<int64_t>(head) * K2 * LB * 64;
#pragma unroll
    for (int kk = 0; kk < K2; ++kk)
#pragma unroll
      for (int lb = 0; lb < LB; ++lb) qb[kk][lb] = src[(kk * LB + lb) * 64 + lane];
  }

  if constexpr ((!COOP && M < 128) || (COOP && WK_LDS)) {  // (not where the accumulators of 128 links need the room)
    // W_V only ever feeds the matrix cores, which read AGPRs as readily as VGPRs: pinned there, it leaves the
    // VGPRs to the values the vector ALUs touch and needs no copies.
#pragma unroll
    for (int kk = 0; kk < K1; ++kk)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) asm volatile("" : "+a"(wv[kk][mb]));
  }
  f32x16 acc[MB][LB];
  float run_max[LB], run_sum[LB];
#pragma unroll
  for (int lb = 0; lb < LB; ++lb) {
    run_max[lb] = -INFINITY;
    run_sum[lb] = 0.f;
#pragma unroll
    for (int ob = 0; ob < MB; ++ob)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[ob][lb][i] = 0.f;
  }

  // COOP: this wave's share of a tile (32 rows = 64 D contiguous bytes), 16 bytes per lane and load
  auto issue = [&](int i0, bf16x8 (&r)[LW]) {
#pragma unroll
    for (int j = 0; j < LW; ++j) {
      const int q = (head * LW + j) * 64 + lane;
      const int item = i0 + q / CPR;
      bf16x8 v;
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = static_cast<__bf16>(0.f);
      if (item < i_end) v = *reinterpret_cast<const bf16x8*>(Eb + static_cast<int64_t>(item) * D + (q % CPR) * 8);
      r[j] = v;
    }
  };

  auto process_tile = [&](int i0, const bf16x8 (&x)[K1]) {
    // The LDS copy of W_K^T must be re-read for every tile (that is the point of keeping it in LDS
    // rather than in registers); an opaque base index stops the compiler from hoisting the reads.
    int wk_base = lane;
    asm volatile("" : "+v"(wk_base));

    f32x16 d1[MB], d2[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) d1[mb][i] = d2[mb][i] = 0.f;
    // the LDS reads run kAhead k-steps ahead of the MFMAs that use them (one wave per SIMD: nobody else
    // covers the LDS latency)
    constexpr int kAhead = 3;
    bf16x8 wkf[WK_LDS ? K1 : 1][MB];
    auto fetch = [&](int kk) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) wkf[WK_LDS ? kk : 0][mb] = lds_wk[wk_base + (kk * MB + mb) * 64];
    };
    if (WK_LDS) {
#pragma unroll
      for (int kk = 0; kk < kAhead && kk < K1; ++kk) fetch(kk);
    }
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) {
      if (WK_LDS && kk + kAhead < K1) fetch(kk + kAhead);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const bf16x8 w = WK_LDS ? wkf[WK_LDS ? kk : 0][mb] : wk[WK_LDS ? 0 : kk][WK_LDS ? 0 : mb];
        d1[mb] = mfma32(w, x[kk], d1[mb]);
        d2[mb] = mfma32(x[kk], wv[kk][mb], d2[mb]);
      }
    }
    bf16x8 kf[K2], vf[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      kf[2 * mb] = pack_half(d1[mb], 0);
      kf[2 * mb + 1] = pack_half(d1[mb], 1);
      vf[mb][0] = pack_half(d2[mb], 0);
      vf[mb][1] = pack_half(d2[mb], 1);
    }

#pragma unroll
    for (int lb = 0; lb < LB; ++lb) {
      f32x16 sc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sc[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K2; ++kk) sc = mfma32(kf[kk], qb[kk][lb], sc);
      // register 4j + r of this lane is item i0 + 8j + 4g + r; only a chunk's last tile can be ragged
      const float c = a.scale * kLog2e;  // >= 0: a negative scale is folded into the sign of the packed queries
      const bool ragged = i0 + 32 > i_end;  // uniform
      if (PHI == kPhiSoftmax) {
        if (ragged) {
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (i0 + 8 * (i >> 2) + 4 * g + (i & 3) >= i_end) sc[i] = -INFINITY;
        }
        float tmax = sc[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, sc[i]);
        tmax = pair_max(tmax);
        const float new_max = fmaxf(run_max[lb], tmax);  // finite: the tile holds at least one valid item
        if (__any(new_max > run_max[lb])) {  // uniform; after the first tiles the maximum rarely moves
          const float alpha = run_max[lb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((run_max[lb] - new_max) * c);
          run_sum[lb] *= alpha;
          run_max[lb] = new_max;
#pragma unroll
          for (int ob = 0; ob < MB; ++ob)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ob][lb][i] *= alpha;
        }
        const float shift = -new_max * c;  // exp2(raw * c + shift) = exp(scale * raw - running maximum)
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float raw = sc[i];
          sc[i] = __builtin_amdgcn_exp2f(fmaf(raw, c, shift));
          if (ragged && raw == -INFINITY) sc[i] = 0.f;  // (explicit: also right for scale = 0)
          psum += sc[i];
        }
        run_sum[lb] += psum;
      } else {
        // SiLU(scale * s) = scale * s * sigmoid(scale * s); the factor `scale` is applied by the merge
#pragma unroll
        for (int i = 0; i < 16; ++i) sc[i] = sc[i] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-sc[i] * c));
        // (no mask is needed here: rows past the end of the chunk were loaded as zeros, so their projected keys are
        // zero, their logits are zero and SiLU(0) = 0 exactly)
      }
      const bf16x8 p0 = pack_half(sc, 0), p1 = pack_half(sc, 1);
#pragma unroll
      for (int ob = 0; ob < MB; ++ob) {
        acc[ob][lb] = mfma32(vf[ob][0], p0, acc[ob][lb]);
        acc[ob][lb] = mfma32(vf[ob][1], p1, acc[ob][lb]);
      }
    }
  };

  if constexpr (COOP) {
    bf16x8 ring[P][LW];
#pragma unroll
    for (int p = 0; p < P; ++p)
      if (i_begin + 32 * p < i_end) issue(i_begin + 32 * p, ring[p]);
    for (int base = i_begin; base < i_end; base += 32 * P) {
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const int i0 = base + 32 * p;
        if (i0 >= i_end) break;  // uniform over the workgroup
        unsigned char* buf = xs[NXS == 2 ? p & 1 : 0];
#pragma unroll
        for (int j = 0; j < LW; ++j) {
          const int q = (head * LW + j) * 64 + lane;
          *reinterpret_cast<bf16x8*>(buf + (q / CPR) * PITCH + (q % CPR) * 16) = ring[p][j];
        }
        // with two buffers a wave arrives here only after it has finished reading the tile before the
        // previous one, which is the one this buffer held; with one, a second barrier follows the reads
        __syncthreads();
        if (i0 + 32 * P < i_end) issue(i0 + 32 * P, ring[p]);
        bf16x8 x[K1];
#pragma unroll
        for (int kk = 0; kk < K1; ++kk) x[kk] = *reinterpret_cast<const bf16x8*>(buf + n * PITCH + 32 * kk + 16 * g);
        if (NXS == 1) __syncthreads();
        process_tile(i0, x);
      }
    }
  } else {
    for (int i0 = i_begin; i0 < i_end; i0 += 32) {
      bf16x8 x[K1];
#pragma unroll
      for (int kk = 0; kk < K1; ++kk) x[kk] = xnext[kk];
      if (i0 + 32 < i_end) load_tile(i0 + 32, xnext);
      process_tile(i0, x);
    }
  }

  // partials: lane (link n of block lb) holds head columns 32ob + 8j + 4g + r in register 4j + r
  const int64_t slot = (static_cast<int64_t>(b) * a.chunks + chunk) * H + head;
#pragma unroll
  for (int lb = 0; lb < LB; ++lb) {
    const int link = 32 * lb + n;
    float* dst = a.part_acc + (slot * M + link) * DH + 4 * g;
#pragma unroll
    for (int ob = 0; ob < MB; ++ob)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float4 v = make_float4(acc[ob][lb][4 * j], acc[ob][lb][4 * j + 1], acc[ob][lb][4 * j + 2], acc[ob][lb][4 * j + 3]);
        *reinterpret_cast<float4*>(dst + 32 * ob + 8 * j) = v;
      }
    const float total = pair_sum(run_sum[lb]);
    if (g == 0) {
      float* ml = a.part_ml + (slot * M + link) * 2;
      ml[0] = run_max[lb] * a.scale;  // the merge works on scaled logits
      ml[1] = total;
    }
  }
}

struct MergeArgs {
  const float* part_acc;
  const float* part_ml;
  const int32_t* lens;
  bf16_t* LP;
  int N, chunk_items, chunks, h, m, dh;
  float scale;  // |logit scale|: the factor the SiLU partials still lack
};

// The merged values LP[b][link][a dh + t .. t + 3] of a user's chunks, combined in ascending order (t is a multiple
// of four: one 16-byte load per chunk serves four outputs, and the load path of a compute unit, not the arithmetic,
// is what this step keeps busy).
template <int PHI>
__device__ __forceinline__ float4 merged_values(const MergeArgs& a, int b, int link, int head, int t, int len) {
  const int used = (len + a.chunk_items - 1) / a.chunk_items;  // chunks that hold at least one valid item
  float4 out = make_float4(0.f, 0.f, 0.f, 0.f);
  if (used > 0) {
    const int64_t stride = static_cast<int64_t>(a.h) * a.m;  // (head, link) slots per chunk
    const int64_t first = (static_cast<int64_t>(b) * a.chunks * a.h + head) * a.m + link;
    // all loads of a batch of chunks are issued before any is used: the partials were written by
    // other compute units and every access is a long-latency miss
    constexpr int kBatch = 16;
    if (PHI == kPhiSoftmax) {
      float gmax = -INFINITY, den = 0.f;
      float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int c0 = 0; c0 < used; c0 += kBatch) {
        float2 ml[kBatch];  // (scaled maximum, sum)
        float4 ac[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
          const int64_t s = first + static_cast<int64_t>(min(c0 + i, used - 1)) * stride;
          ml[i] = *reinterpret_cast<const float2*>(a.part_ml + s * 2);
          ac[i] = *reinterpret_cast<const float4*>(a.part_acc + s * a.dh + t);
        }
        float bmax = gmax;
#pragma unroll
        for (int i = 0; i < kBatch; ++i) bmax = fmaxf(bmax, ml[i].x);
        const float keep = __builtin_amdgcn_exp2f((gmax - bmax) * kLog2e);  // 0 on the first batch
        num.x *= keep, num.y *= keep, num.z *= keep, num.w *= keep;
        den *= keep;
        gmax = bmax;
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
          const float w = c0 + i < used ? __builtin_amdgcn_exp2f((ml[i].x - gmax) * kLog2e) : 0.f;
          num.x = fmaf(w, ac[i].x, num.x), num.y = fmaf(w, ac[i].y, num.y);
          num.z = fmaf(w, ac[i].z, num.z), num.w = fmaf(w, ac[i].w, num.w);
          den = fmaf(w, ml[i].y, den);
        }
      }
      out = make_float4(num.x / den, num.y / den, num.z / den, num.w / den);
    } else {
      float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int c0 = 0; c0 < used; c0 += kBatch) {
        float4 ac[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i)
          ac[i] = *reinterpret_cast<const float4*>(
              a.part_acc + (first + static_cast<int64_t>(min(c0 + i, used - 1)) * stride) * a.dh + t);
#pragma unroll
        for (int i = 0; i < kBatch; ++i)
          if (c0 + i < used) num.x += ac[i].x, num.y += ac[i].y, num.z += ac[i].z, num.w += ac[i].w;
      }
      const float f = a.scale / static_cast<float>(len);
      out = make_float4(num.x * f, num.y * f, num.z * f, num.w * f);
    }
  }
  return out;
}

// Four rounded link-state values as one 8-byte store.
__device__ __forceinline__ void store_rounded(bf16_t* dst, const float4& v, float* rounded = nullptr) {
  alignas(8) bf16_t r[4];
  store_as(&r[0], v.x), store_as(&r[1], v.y), store_as(&r[2], v.z), store_as(&r[3], v.w);
  *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(r);
  if (rounded != nullptr)
    *reinterpret_cast<float4*>(rounded) = make_float4(to_float(r[0]), to_float(r[1]), to_float(r[2]), to_float(r[3]));
}

// One thread per four adjacent output elements LP[b][link][a dh + t .. t + 3], one wave per workgroup: the
// workgroups spread over as many compute units as there are.
constexpr int kMergeThreads = 64;
template <int PHI>
__global__ __launch_bounds__(kMergeThreads) void merge_kernel(MergeArgs a) {
  const int b = blockIdx.y;
  const int idx = (blockIdx.x * kMergeThreads + threadIdx.x) * 4;
  const int d = a.h * a.dh;
  if (idx >= a.m * d) return;
  const int link = idx / d, col = idx % d, head = col / a.dh, t = col % a.dh;
  const int len = a.lens ? min(a.lens[b], a.N) : a.N;
  store_rounded(a.LP + (static_cast<int64_t>(b) * a.m + link) * d + col, merged_values<PHI>(a, b, link, head, t, len));
}

// Merge and the candidate stage's value projection in one kernel: a block finishes kMvRows link states of one user
// (four adjacent elements per thread, as the merge kernel does), stores them, and projects their bf16-rounded values onto Wv:
// V~ = LP Wv, written as the value image (kPackValues) that the candidate-side kernel loads.  Same split of the sum
// over d as the pack kernel's projections: thread (cg, kc) owns 8 adjacent columns and every nkc-th k; the partial
// sums meet in LDS.  Every partial state is read once, as in the merge kernel: those reads miss the local L2
// (other compute units wrote them) and set the kernel's time.
// The workgroup has 2 d threads: d / 8 column groups x 16 k-groups (d / 16 k-steps per thread), of which d / 2
// threads do the merge.
constexpr int kMvRows = 2, kMvKGroups = 16;
struct MergeValuesArgs {
  MergeArgs m;
  const bf16_t* Wv;  // [d][d], nullable = identity
  bf16_t* VA;        // [B] value images
  int passes;        // row pairs a workgroup handles one after the other with the same W_V registers
  // layer normalisation of the finished link states before the projection (ln_on; LP is stored un-normalised)
  const bf16_t *ln_gamma, *ln_beta;
  float ln_eps;
  int ln_on;
};

template <int PHI, int D>
__global__ __launch_bounds__(2 * D) void merge_values_kernel(MergeValuesArgs a) {
  constexpr int d = D, kMvThreads = 2 * D, CG = D / 8, nkc = kMvKGroups, kMvMaxK = D / kMvKGroups;
  static_assert(CG * nkc == kMvThreads, "one thread per (column group, k-group)");
  // rounded link states + output rows + one partial output per k-group (36 KiB at d = 256)
  __shared__ float lp[kMvRows * D];         // bf16-rounded values
  __shared__ float out[kMvRows * D];
  // (a column c sits at c + c / 32: the writers' columns are 8 apart, which would otherwise share four banks)
  constexpr int kRedRow = D + D / 32;
  __shared__ float red[nkc * kMvRows * kRedRow];
  const int tid = threadIdx.x, b = blockIdx.y;
  const int cg = tid % CG, kc = tid / CG;
  bf16x8 wreg[kMvMaxK];
  if (a.Wv != nullptr) {  // asked for before the merge, used after it
#pragma unroll
    for (int it = 0; it < kMvMaxK; ++it)
      wreg[it] = *reinterpret_cast<const bf16x8*>(a.Wv + static_cast<int64_t>(kc + it * nkc) * d + 8 * cg);
  }
  constexpr int kLnWaves = kMvThreads / 64, kLnPerLane = (D + 63) / 64;
  const int len = a.m.lens ? min(a.m.lens[b], a.m.N) : a.m.N;
  // (no barrier is needed between two passes: whoever writes lp, red or out again has passed two barriers since
  // the last read of it)
  const int passes = D >= 256 ? a.passes : 1;  // (a compile-time 1 keeps the small shapes' register count low)
  for (int pass = 0; pass < passes; ++pass) {
    const int row0 = (blockIdx.x * passes + pass) * kMvRows;
    for (int i = 4 * tid; i < kMvRows * d; i += 4 * kMvThreads) {
      const int link = row0 + i / d, col = i % d;
      store_rounded(a.m.LP + (static_cast<int64_t>(b) * a.m.m + link) * d + col,
                    merged_values<PHI>(a.m, b, link, col / a.m.dh, col % a.m.dh, len), lp + i);
    }
    __syncthreads();
    if (a.ln_on) {  // uniform
      // a wavefront per row: mean, centred second moment, then the normalised row rounded to bf16, as a
      // normalisation pass of its own would have stored it
      // (the thread index through an opaque copy: what is derived from it here - addresses, the scale and the shift -
      // is then computed and fetched here, not ahead of the merge, which has no registers to carry it and would
      // spill; the fetches are in flight during the two reductions)
      int t_ln = tid;
      asm volatile("" : "+v"(t_ln));
      for (int r = t_ln / 64; r < kMvRows; r += kLnWaves) {
        float* xr = lp + r * d;
        bf16_t ln_g[kLnPerLane], ln_b[kLnPerLane];
#pragma unroll
        for (int i = 0; i < kLnPerLane; ++i) {
          const int k = min(t_ln % 64 + 64 * i, d - 1);
          ln_g[i] = a.ln_gamma[k], ln_b[i] = a.ln_beta[k];
        }
        float x[kLnPerLane], sum = 0.f;
#pragma unroll
        for (int i = 0; i < kLnPerLane; ++i) {
          const int k = t_ln % 64 + 64 * i;
          x[i] = k < d ? xr[k] : 0.f;
          sum += x[i];
        }
        const float mean = wave_sum(sum) * (1.f / d);
        float q = 0.f;
#pragma unroll
        for (int i = 0; i < kLnPerLane; ++i) {
          const int k = t_ln % 64 + 64 * i;
          x[i] = k < d ? x[i] - mean : 0.f;
          q = fmaf(x[i], x[i], q);
        }
        const float inv = 1.f / sqrtf(wave_sum(q) * (1.f / d) + a.ln_eps);
#pragma unroll
        for (int i = 0; i < kLnPerLane; ++i) {
          const int k = t_ln % 64 + 64 * i;
          if (k < d) xr[k] = static_cast<float>(static_cast<__bf16>(fmaf(x[i] * inv, to_float(ln_g[i]), to_float(ln_b[i]))));
        }
      }
      __syncthreads();
    }
    if (a.Wv == nullptr) {
      for (int i = tid; i < kMvRows * d; i += kMvThreads) out[i] = lp[i];
    } else {
      float acc[kMvRows][8];
#pragma unroll
      for (int r = 0; r < kMvRows; ++r)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[r][j] = 0.f;
#pragma unroll
      for (int it = 0; it < kMvMaxK; ++it) {
#pragma unroll
        for (int r = 0; r < kMvRows; ++r) {
          const float x = lp[r * d + kc + it * nkc];
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[r][j] = fmaf(x, static_cast<float>(wreg[it][j]), acc[r][j]);
        }
      }
#pragma unroll
      for (int r = 0; r < kMvRows; ++r)
#pragma unroll
        for (int j = 0; j < 8; ++j) red[(kc * kMvRows + r) * kRedRow + 8 * cg + j + (cg >> 2)] = acc[r][j];
      __syncthreads();
      for (int i = tid; i < kMvRows * d; i += kMvThreads) {
        float sum = 0.f;
#pragma unroll 8
        for (int c = 0; c < nkc; ++c) sum += red[(c * kMvRows + i / d) * kRedRow + i % d + (i % d) / 32];
        out[i] = sum;
      }
    }
    __syncthreads();
    for (int i = tid; i < kMvRows * d; i += kMvThreads)
      store_as(a.VA + values_slot(b, row0 + i / d, i % d, d, a.m.dh, a.m.m, true), out[i]);
  }
}

template <int DH, int M, int H, int PHI>
hipError_t launch_phi(const HistArgs& a, int users, bool coop, hipStream_t s) {
  constexpr bool kWkLds = DH * H >= 256;
  constexpr size_t slice = kWkLds ? static_cast<size_t>(DH) * H * DH * 2 : 0;  // one head's slice of W_K^T
  if constexpr (H > 1 && !(kWkLds && H > 4)) {  // (eight waves of d = 256 would not fit the register file)
    if (coop) {
      constexpr size_t lds = slice * H;
      auto kernel = links_over_history_kernel<DH, M, H, PHI, kWkLds, true>;
      if (lds > 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (attr != hipSuccess) return attr;
      }
      launch_timed(kKernelLinksOverHistory, kernel, dim3(a.chunks, users), dim3(64 * H), lds, s, a);
      return hipGetLastError();
    }
  }
  auto kernel = links_over_history_kernel<DH, M, H, PHI, kWkLds, false>;
  if (slice > 64 * 1024) {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(slice));
    if (attr != hipSuccess) return attr;
  }
  launch_timed(kKernelLinksOverHistory, kernel, dim3(a.chunks, users, H), dim3(64), slice, s, a);
  return hipGetLastError();
}

template <int DH, int M, int H>
hipError_t launch_main(const HistArgs& a, int phi, int users, bool coop, hipStream_t s) {
  return phi == kPhiSoftmax ? launch_phi<DH, M, H, kPhiSoftmax>(a, users, coop, s)
                            : launch_phi<DH, M, H, kPhiSilu>(a, users, coop, s);
}

template <int DH, int H>
hipError_t dispatch_m(const HistArgs& a, int links, int phi, int users, bool coop, hipStream_t s) {
  switch (links) {
    case 32: return launch_main<DH, 32, H>(a, phi, users, coop, s);
    case 64: return launch_main<DH, 64, H>(a, phi, users, coop, s);
    case 96: return launch_main<DH, 96, H>(a, phi, users, coop, s);
    case 128: return launch_main<DH, 128, H>(a, phi, users, coop, s);
  }
  return hipErrorInvalidValue;
}

template <int DH>
hipError_t dispatch_h(const HistArgs& a, int h, int links, int phi, int users, bool coop, hipStream_t s) {
  switch (h) {
    case 1: return dispatch_m<DH, 1>(a, links, phi, users, coop, s);
    case 2: return dispatch_m<DH, 2>(a, links, phi, users, coop, s);
    case 4: return dispatch_m<DH, 4>(a, links, phi, users, coop, s);
    case 8: if (DH == 32) return dispatch_m<32, 8>(a, links, phi, users, coop, s);
  }
  return hipErrorInvalidValue;
}

struct Layout {
  int chunk_items, chunks;
  bool coop;  // h-wave workgroups that stage each tile once through LDS (long histories, d <= 128)
  size_t wk, wv, qb, acc, ml, total;
};

Layout plan(int B, int N, int d, int h, int m, bool q_per_user) {
  Layout l{};
  const int tiles = (N + 31) / 32;
  // Short histories: every (chunk, head) pair is a one-wave workgroup and a compute unit runs four of
  // them at once (eight when d/h = 32); aim at one round of workgroups.  Long histories with d <= 128
  // (at least four tiles per compute unit): h-wave workgroups, two per compute unit.  At least two
  // tiles per chunk so that the stationary operands are fetched for more than one tile and the merge
  // stays small.
  l.coop = h > 1 && !(d >= 256 && h > 4) && static_cast<int64_t>(B) * tiles >= 4 * static_cast<int64_t>(compute_units());
  // (at d = 256 the cooperative workgroup keeps all of W_K^T in LDS and is alone on its compute unit)
  const int64_t slots = static_cast<int64_t>(l.coop ? (d >= 256 ? 1 : 2) : (d / h == 32 ? 8 : 4)) * compute_units();
  int chunk_tiles = static_cast<int>((static_cast<int64_t>(B) * tiles * (l.coop ? 1 : h) + slots - 1) / slots);
  if (chunk_tiles < 2) chunk_tiles = 2;
  if (chunk_tiles > tiles) chunk_tiles = tiles;
  l.chunk_items = chunk_tiles * 32;
  l.chunks = (tiles + chunk_tiles - 1) / chunk_tiles;
  l.wk = l.wv = align_up(static_cast<size_t>(d) * d * 2);
  l.qb = align_up(static_cast<size_t>(q_per_user ? B : 1) * m * d * 2);
  l.acc = align_up(static_cast<size_t>(B) * l.chunks * m * d * sizeof(float));
  l.ml = align_up(static_cast<size_t>(B) * l.chunks * h * m * 2 * sizeof(float));
  l.total = l.wk + l.wv + l.qb + l.acc + l.ml;
  return l;
}

}  // namespace

bool links_over_history_supported(int d, int h, int m) { return queries_over_links_supported(d, h, m); }

size_t links_over_history_workspace(int B, int N, int d, int h, int m, bool q_per_user) {
  return plan(B, N, d, h, m, q_per_user).total;
}

void links_over_history_jobs(const LinksOverHistory& q, void* workspace, PackJobs& jobs) {
  const Layout l = plan(q.B, q.N, q.d, q.h, q.m, q.lc_user_stride != 0);
  char* ws = static_cast<char*>(workspace);
  jobs.weights[jobs.n_weights++] = PackWeight{q.Wk, ws};
  jobs.weights[jobs.n_weights++] = PackWeight{q.Wv, ws + l.wk};
  // a negative logit scale is folded into the sign of the packed queries, so the kernels see scale >= 0
  jobs.projections[jobs.n_projections++] = PackProject{q.LC, q.Wq, ws + l.wk + l.wv, q.lc_user_stride,
                                                       q.lc_user_stride != 0 ? q.B : 1, kPackKeys, q.scale < 0.f ? -1.f : 1.f, q.q_norm};
}

hipError_t links_over_history(const LinksOverHistory& q, void* workspace, hipStream_t s) {
  const int d = q.d, h = q.h, m = q.m, dh = d / h;
  const bool per_user = q.lc_user_stride != 0;
  const Layout l = plan(q.B, q.N, d, h, m, per_user);
  char* ws = static_cast<char*>(workspace);
  void* WkA = ws;
  void* WvB = ws + l.wk;
  void* QB = ws + l.wk + l.wv;
  float* part_acc = reinterpret_cast<float*>(ws + l.wk + l.wv + l.qb);
  float* part_ml = reinterpret_cast<float*>(ws + l.wk + l.wv + l.qb + l.acc);

  hipError_t e = hipSuccess;
  if (q.prepared != nullptr) {  // nothing to pack
    const PreparedLayout pl = prepared_layout(d, m);
    char* base = const_cast<char*>(static_cast<const char*>(q.prepared));
    WkA = base + pl.wk, WvB = base + pl.wv, QB = base + pl.qb;
  } else if (!q.packed) {
    PackJobs jobs;
    links_over_history_jobs(q, workspace, jobs);
    e = pack_operands(jobs, d, h, m, s);
    if (e != hipSuccess) return e;
  }

  HistArgs a{};
  a.E = static_cast<const bf16_t*>(q.E), a.lens = q.lens;
  a.WkA = static_cast<const bf16x8*>(WkA), a.WvB = static_cast<const bf16x8*>(WvB);
  a.QB = static_cast<const bf16x8*>(QB);
  a.qb_user_frags = per_user ? static_cast<int64_t>(m) * d / 8 : 0;
  a.part_acc = part_acc, a.part_ml = part_ml;
  a.N = q.N, a.chunk_items = l.chunk_items, a.chunks = l.chunks, a.scale = fabsf(q.scale);
  e = dh == 32 ? dispatch_h<32>(a, h, m, q.phi, q.B, l.coop, s) : dispatch_h<64>(a, h, m, q.phi, q.B, l.coop, s);
  if (e != hipSuccess) return e;

  MergeArgs g{part_acc, part_ml, q.lens, static_cast<bf16_t*>(q.LP), q.N, l.chunk_items, l.chunks, h, m, dh, fabsf(q.scale)};
  if (q.values_image != nullptr) {
    // With many users and the largest W_V a workgroup takes several row pairs in turn, as long as every compute
    // unit still has a workgroup: each workgroup reads all of W_V (128 KiB at d = 256; at d = 128 the shorter
    // chain per workgroup is worth more than the 32 KiB: measured).
    int passes = 1;
    while (d >= 256 && passes < 16 && static_cast<int64_t>(q.B) * (m / kMvRows) / (2 * passes) >= compute_units())
      passes *= 2;
    MergeValuesArgs mv{g, static_cast<const bf16_t*>(q.Wv_values), static_cast<bf16_t*>(q.values_image), passes,
                       static_cast<const bf16_t*>(q.values_norm.gamma), static_cast<const bf16_t*>(q.values_norm.beta),
                       q.values_norm.eps, q.values_norm.on ? 1 : 0};
    const dim3 vgrid(m / (kMvRows * passes), q.B);  // (m / 2 is a multiple of 16)
    const bool softmax = q.phi == kPhiSoftmax;
#define LIME_MV_CASE(D)                                                                                      \
  case D:                                                                                                    \
    if (softmax)                                                                                             \
      hipLaunchKernelGGL((merge_values_kernel<kPhiSoftmax, D>), vgrid, dim3(2 * D), 0, s, mv);               \
    else                                                                                                     \
      hipLaunchKernelGGL((merge_values_kernel<kPhiSilu, D>), vgrid, dim3(2 * D), 0, s, mv);                  \
    break;
    switch (d) {  // every d the matrix-core kernels take
      LIME_MV_CASE(32)
      LIME_MV_CASE(64)
      LIME_MV_CASE(128)
      LIME_MV_CASE(256)
      default:
        return hipErrorInvalidValue;
    }
#undef LIME_MV_CASE
    return hipGetLastError();
  }
  const dim3 mgrid((m * d / 4 + kMergeThreads - 1) / kMergeThreads, q.B);
  if (q.phi == kPhiSoftmax)
    hipLaunchKernelGGL(merge_kernel<kPhiSoftmax>, mgrid, dim3(kMergeThreads), 0, s, g);
  else
    hipLaunchKernelGGL(merge_kernel<kPhiSilu>, mgrid, dim3(kMergeThreads), 0, s, g);
  return hipGetLastError();
}

}  // namespace lime
