// Candidate-side decoupled attention (Eq. 4) on the matrix cores, and with phi = SiLU/m the
// history-to-links direction O[S] of XORA (Eq. 7).
//
// Design: weights stationary in registers, query rows streamed.  A workgroup has one wavefront
// per head.  Wave a keeps, as MFMA A-operand fragments in its registers, the head-a slices of
// W_Q^T (d/h x d), of the projected keys K~ (m x d/h) and of the projected values V~^T (d/h x m).
// For each tile of 32 query rows it chains three contractions without leaving registers:
//   Q~^T (d/h x 32) = W_Q,a^T  . X^T        X rows are the B operand (staged once per tile through LDS)
//   S^T  (m   x 32) = K~_a     . Q~^T       B operand = the accumulators of the first product
//   O^T  (d/h x 32) = V~_a^T   . phi(S)^T   B operand = the accumulators of the second product
// Every lane owns one query row (column of the transposed products), so the softmax over the m
// links is a reduction over the lane's own registers plus one exchange with lane ^ 32.
// A small pack kernel computes K~ = Ksrc Wk and V~ = Vsrc Wv once per call and lays all three
// stationary operands out in fragment order, so the main kernel loads them with 16-byte accesses.
//
// FUSED: when the keys are the same for every user (the candidate side of LIME: links and weights are model
// parameters, Section 3.3) and there are no more links than head columns, the first two products collapse into
//   S^T  (m   x 32) = G_a^T    . X^T,       G_a = W_Q,a K~_a^T  (d x m), built once per model by lime_prepare,
// which saves the second product, the bf16 rounding of Q~ and the registers of K~.
#include <type_traits>

#include "mfma.hpp"

namespace lime {
namespace {

constexpr float kLog2e = 1.4426950408889634f;

// ----------------------------------------------------------------------------- main kernel
struct MainArgs {
  const bf16_t* X;
  bf16_t* O;
  const bf16x8 *WqA, *KA, *VA;  // FUSED: WqA is the image of G and KA is unused
  int64_t ka_user_frags, va_user_frags;  // fragment-image size per user (0 = shared), in bf16x8 units
  const int32_t* row_lens;
  int B, rows, tiles_per_user, total_tiles;
  float scale, inv_norm;
  bf16_t* Wout;  // WEIGHTS variant only
  bool fused;
  // NORM variant only: layer normalisation of the query rows (gamma, beta nullable = 1, 0)
  const bf16_t *ln_gamma, *ln_beta;
  float ln_eps;
  bool ln_on;
};

// WEIGHTS: stop after phi and write the normalised attention weights [rows][h][m] (the QK cache of
// Section 3.3) instead of the weighted sum.
// NORM: the query rows are layer-normalised over their d features (Appendix C) on their way from the register ring
// into LDS: a row is 16 bytes in each of d/8 neighbouring lanes of one load, so its statistics are a few lane
// exchanges, and every element is handled once per tile whichever waves read it afterwards.  Rounded to bf16 where
// a normalisation pass of its own would have stored the row.
template <int DH, int M, int H, int PHI, bool WEIGHTS, bool FUSED, bool NORM = false>
__global__ __launch_bounds__(64 * H) void queries_over_links_kernel(MainArgs a) {
  constexpr int D = DH * H;
  constexpr int K1 = D / 16, MB = DH / 32;   // first product: k-steps over d, row blocks over d/h
  constexpr int K2 = DH / 16, LB = M / 32;   // second: k-steps over d/h, row blocks over links
  constexpr int FB = FUSED ? LB : MB;        // row blocks of the first product (FUSED: over links)
  constexpr int K3 = M / 16;                 // third: k-steps over links, row blocks over d/h (MB)
  // A tile is 32 consecutive rows of X = 64 D contiguous bytes.  The H waves copy it cooperatively:
  // each wave issues LW loads of 1 KiB (16 bytes per lane, fully coalesced) into a register ring that
  // keeps P tiles in flight per workgroup (besides the two tiles parked in LDS), then parks the tile in
  // LDS (row pitch padded by 16 bytes so that the fragment reads are free of bank conflicts) where all
  // H waves read it.
  constexpr int P = 2;
  constexpr int LW = DH / 16;
  // With d = 256 the W_Q^T slice alone is a quarter of the register file; with many links (whose
  // logits and weights need registers too) the second half of its k-steps lives in LDS instead and is
  // read once per tile, which keeps the kernel free of register spills.
  // (eight heads: eight waves share the register file two to a SIMD, so with many links three quarters go there)
  constexpr int KL = D < 256 ? 0 : H == 8 ? (M >= 96 ? 3 * K1 / 4 : 0) : (M >= 128 ? K1 / 2 : 0);  // k-steps of W_Q^T kept in LDS
  static_assert(!FUSED || (KL == 0 && M <= DH), "the fused form is for few links");
  constexpr int KR = K1 - KL;                // k-steps kept in registers
  constexpr int CPR = D / 8;            // 16-byte chunks per row of X
  constexpr int PITCH = 2 * D + 16;     // LDS row pitch of an X tile, bytes
  constexpr int OCPR = DH / 8;          // 16-byte chunks per row of one head's output slice
  constexpr int OPITCH = 2 * DH + 16;   // LDS row pitch of a wave's output tile, bytes
  __shared__ __attribute__((aligned(16))) unsigned char xs[2][32 * PITCH];
  __shared__ __attribute__((aligned(16))) unsigned char os[H][32 * OPITCH];
  __shared__ bf16x8 wq_lds[KL > 0 ? H * KL * FB * 64 : 1];
  const int lane = threadIdx.x & 63, head = threadIdx.x >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int64_t total_rows = static_cast<int64_t>(a.B) * a.rows;
  // Each workgroup owns a contiguous run of tiles (neighbouring rows share pages and DRAM rows).
  const int per_wg = (a.total_tiles + gridDim.x - 1) / gridDim.x;
  const int first = blockIdx.x * per_wg;
  const int last = min(first + per_wg, a.total_tiles);  // one past this workgroup's final tile
  if (first >= last) return;  // uniform

  // Rows past a user's last row are read from whatever follows (the next user's rows; zeros past the
  // end of the tensor): every row is an independent column of the three products and such columns
  // are never stored.
  // A tile is named by (user, first row); the byte offsets of a lane's pieces inside a tile never change,
  // so that a load is one scalar base plus a per-lane offset.
  int xoff[LW], ooff[LW];
#pragma unroll
  for (int j = 0; j < LW; ++j) {
    const int q = (head * LW + j) * 64 + lane;
    xoff[j] = ((q / CPR) * D + (q % CPR) * 8) * 2;
    const int o = j * 64 + lane;
    ooff[j] = ((o / OCPR) * D + (o % OCPR) * 8) * 2;
  }
  auto issue = [&](int tb, int tr0, bf16x8 (&r)[LW]) {
    const int64_t row0 = static_cast<int64_t>(tb) * a.rows + tr0;
    const unsigned char* base = reinterpret_cast<const unsigned char*>(a.X) + row0 * (2 * D);
    if (row0 + 32 <= total_rows) {  // uniform: the whole tile lies inside the tensor
#pragma unroll
      for (int j = 0; j < LW; ++j) r[j] = *reinterpret_cast<const bf16x8*>(base + xoff[j]);
    } else {
#pragma unroll
      for (int j = 0; j < LW; ++j) {
        const int q = (head * LW + j) * 64 + lane;
        bf16x8 v;
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = static_cast<__bf16>(0.f);
        if (row0 + q / CPR < total_rows) v = *reinterpret_cast<const bf16x8*>(base + xoff[j]);
        r[j] = v;
      }
    }
  };
  // (user, first row) of a tile index, and of the tile after a given one
  auto locate = [&](int tile, int& tb, int& tr0) {
    tb = tile / a.tiles_per_user;
    tr0 = (tile - tb * a.tiles_per_user) * 32;
  };
  auto advance = [&](int& tb, int& tr0) {
    tr0 += 32;
    if (tr0 >= a.rows) tr0 = 0, ++tb;
  };
  // NORM: scale and shift of this lane's eight columns (the same in every tile), asked for ahead of everything else
  bf16x8 ln_gv, ln_bv;
  if constexpr (NORM) {
    ln_gv = *reinterpret_cast<const bf16x8*>(a.ln_gamma + 8 * (lane % CPR));
    ln_bv = *reinterpret_cast<const bf16x8*>(a.ln_beta + 8 * (lane % CPR));
  }
  auto normalised = [&](const bf16x8& v) -> bf16x8 {
    float x[8], sum = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) x[t] = static_cast<float>(v[t]), sum += x[t];
    sum = group_sum<CPR>(sum);
    const float mean = sum * (1.f / D);
    float q = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) x[t] -= mean, q = fmaf(x[t], x[t], q);
    q = group_sum<CPR>(q);
    const float inv = __builtin_amdgcn_rsqf(q * (1.f / D) + a.ln_eps);
    bf16x8 y;
#pragma unroll
    for (int t = 0; t < 8; ++t) y[t] = static_cast<__bf16>(fmaf(x[t] * inv, static_cast<float>(ln_gv[t]), static_cast<float>(ln_bv[t])));
    return y;
  };
  auto park = [&](const bf16x8 (&r)[LW], unsigned char* buf) {
#pragma unroll
    for (int j = 0; j < LW; ++j) {
      const int q = (head * LW + j) * 64 + lane;
      bf16x8* dst = reinterpret_cast<bf16x8*>(buf + (q / CPR) * PITCH + (q % CPR) * 16);
      if constexpr (NORM) *dst = normalised(r[j]);
      else *dst = r[j];
    }
  };

  bf16x8 ring[P][LW];
  int ib, ir0;  // the next tile to request
  locate(first, ib, ir0);
  const int b_first = ib, r0_first = ir0;
#pragma unroll
  for (int p = 0; p < P; ++p)
    if (first + p < last) {
      issue(ib, ir0, ring[p]);
      advance(ib, ir0);
    }

  // A wave's vector memory instructions issue in program order, and the compute unit's address path takes a
  // 16-byte-per-lane load of a wave in 16 cycles: asked for up front, the 50-odd loads of the stationary
  // operands of four waves hold every wave for 1.5 us before it reaches the first use of the first of them.
  // Where all of W_Q^T lives in registers (kJit) the prologue therefore asks for the first tiles and kLead
  // k-steps of W_Q^T only, and feeds the remaining requests (W_Q^T, then K~, then V~^T: the order of their
  // first use) between the matrix instructions of the first tile's first product.
  constexpr bool kJit = KL == 0;
  constexpr int kLead = KR < 4 ? KR : 4;
  bf16x8 wq[KR][FB];
  auto load_wq_step = [&](int kk) {
#pragma unroll
    for (int mb = 0; mb < FB; ++mb) wq[kk][mb] = a.WqA[((head * K1 + kk) * FB + mb + head * kQueryImageHeadPad) * 64 + lane];
  };
  // Otherwise: every workgroup wants the same W_Q^T fragments; asked for in the same order by all compute units
  // at once, the requests queue up at one cache channel after another.  The workgroups of an XCD (consecutive
  // workgroups go to different XCDs) therefore start at different k-steps.  The destination registers and the
  // order of the products stay the same: kRot copies of the load sequence, chosen by a uniform switch.
  constexpr int kRot = !kJit && KR >= 8 ? 4 : 1;
  auto load_wq = [&](auto rot_tag) {
    constexpr int start = decltype(rot_tag)::value * (KR / kRot);
#pragma unroll
    for (int i = 0; i < KR; ++i) {
      const int kk = (i + start) % KR;
#pragma unroll
      for (int mb = 0; mb < FB; ++mb) wq[kk][mb] = a.WqA[((head * K1 + kk) * FB + mb + head * kQueryImageHeadPad) * 64 + lane];
    }
  };
  if constexpr (kJit) {
#pragma unroll
    for (int kk = 0; kk < kLead && kk < KR; ++kk) load_wq_step(kk);
  } else {
    switch (kRot == 1 ? 0 : (blockIdx.x / 8) % kRot) {
      case 1: load_wq(std::integral_constant<int, 1>{}); break;
      case 2: load_wq(std::integral_constant<int, 2>{}); break;
      case 3: load_wq(std::integral_constant<int, 3>{}); break;
      default: load_wq(std::integral_constant<int, 0>{}); break;
    }
  }
  if constexpr (KL > 0) {
    bf16x8 tmp[KL * FB];
#pragma unroll
    for (int i = 0; i < KL * FB; ++i) tmp[i] = a.WqA[((head * K1 + KR) * FB + i + head * kQueryImageHeadPad) * 64 + lane];
#pragma unroll
    for (int i = 0; i < KL * FB; ++i) wq_lds[(head * KL * FB + i) * 64 + lane] = tmp[i];
    // each wave reads back only what it wrote itself: no barrier needed
  }

  // Q~^T = Wq_a^T X^T for the tile parked in `buf`; lane (n, g) reads X[row n][16kk + 8g ..].
  // Fragment reads run kAhead k-steps ahead of the MFMAs that use them (one wave per SIMD: nobody else
  // covers the LDS latency).  first_begin() clears the accumulators and starts the reads, first_mfma(i)
  // issues MFMA i of the K1 * FB, so that the caller can put other work between them.
  f32x16 acc1[FB];
  constexpr int kAhead = 3;
  constexpr int NM = K1 * FB;
  bf16x8 xq[K1], wl_frag[KL > 0 ? KL : 1][FB];
  const unsigned char* xrow = nullptr;
  int wl = 0;
  auto fetch = [&](int kk) {
    xq[kk] = *reinterpret_cast<const bf16x8*>(xrow + 32 * kk);
    if (kk >= KR) {
#pragma unroll
      for (int mb = 0; mb < FB; ++mb) wl_frag[KL > 0 ? kk - KR : 0][mb] = wq_lds[wl + ((kk - KR) * FB + mb) * 64];
    }
  };
  auto first_begin = [&](const unsigned char* buf) {
    xrow = buf + n * PITCH + 16 * g;
#pragma unroll
    for (int mb = 0; mb < FB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc1[mb][i] = 0.f;
    wl = head * KL * FB * 64 + lane;
    asm volatile("" : "+v"(wl));  // keeps the LDS reads of W_Q^T inside the tile loop
#pragma unroll
    for (int kk = 0; kk < kAhead && kk < K1; ++kk) fetch(kk);
  };
  auto first_mfma = [&](int i) {
    const int kk = i / FB, mb = i % FB;
    if (mb == 0 && kk + kAhead < K1) fetch(kk + kAhead);
    const bf16x8 w = kk < KR ? wq[kk < KR ? kk : 0][mb] : wl_frag[kk >= KR ? kk - KR : 0][mb];
    acc1[mb] = mfma32(w, xq[kk], acc1[mb]);
  };
  auto first_product = [&](const unsigned char* buf) {
    first_begin(buf);
#pragma unroll
    for (int i = 0; i < NM; ++i) first_mfma(i);
  };

  // phi over the m links of this lane's query row (the other half of the links sits in lane ^ 32), cut
  // into steps so that the tile loop can put one matrix instruction of the next tile between them:
  // softmax = kMaxSteps partial maxima, the exchange with lane ^ 32, then one step per pair of links
  // (exponential, running sum, bf16 rounding into the B fragments `pf` of the third product).
  // phi_finish() returns the factor still owed to the weighted sum.
  f32x16 acc2[LB];
  bf16x8 pf[K3];
  constexpr int kPairs = LB * 8;
  constexpr int kMaxSteps = PHI == kPhiSoftmax ? LB * 2 : 0;
  constexpr int kPairStep0 = PHI == kPhiSoftmax ? kMaxSteps + 1 : 0;
  constexpr int NV = kPairStep0 + kPairs;
  const float phi_c = a.scale * kLog2e;  // >= 0
  float phi_mx = 0.f, phi_shift = 0.f, phi_sum = 0.f;
  auto phi_step = [&](int st) {
    if (PHI == kPhiSoftmax && st < kMaxSteps) {
      const int lb = st / 2, i0 = (st % 2) * 8;
      if (st == 0) phi_mx = acc2[0][0];
#pragma unroll
      for (int i = 0; i < 8; ++i) phi_mx = fmaxf(phi_mx, acc2[lb][i0 + i]);
    } else if (PHI == kPhiSoftmax && st == kMaxSteps) {
      phi_mx = pair_max(phi_mx);
    } else if (st >= kPairStep0) {
      const int e = st - kPairStep0, lb = e / 8, i = (e % 8) * 2;
      float p0, p1;
      if (PHI == kPhiSoftmax) {
        if (e == 0) {
          phi_shift = -phi_mx * phi_c;  // exp2(raw * c + shift) = exp(scale * raw - max scaled logit)
          phi_sum = 0.f;
        }
        p0 = __builtin_amdgcn_exp2f(fmaf(acc2[lb][i], phi_c, phi_shift));
        p1 = __builtin_amdgcn_exp2f(fmaf(acc2[lb][i + 1], phi_c, phi_shift));
        phi_sum += p0;
        phi_sum += p1;
      } else {
        // SiLU(scale * s) = scale * s * sigmoid(scale * s); `scale` is part of the final factor
        p0 = acc2[lb][i] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-acc2[lb][i] * phi_c));
        p1 = acc2[lb][i + 1] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-acc2[lb][i + 1] * phi_c));
      }
      acc2[lb][i] = p0, acc2[lb][i + 1] = p1;
      pf[2 * lb + (i >> 3)][i & 7] = static_cast<__bf16>(p0);
      pf[2 * lb + (i >> 3)][(i & 7) + 1] = static_cast<__bf16>(p1);
    }
  };
  auto phi_finish = [&]() -> float {
    if (PHI == kPhiSoftmax) return 1.f / pair_sum(phi_sum);
    return a.inv_norm * a.scale;
  };

  bf16x8 ka[K2][LB], va[K3][MB];
  auto load_user = [&](int b, bool keys, bool values) {
    if (keys) {
      const bf16x8* src = a.KA + b * a.ka_user_frags + static_cast<int64_t>(head) * K2 * LB * 64;
#pragma unroll
      for (int kk = 0; kk < K2; ++kk)
#pragma unroll
        for (int lb = 0; lb < LB; ++lb) ka[kk][lb] = src[(kk * LB + lb) * 64 + lane];
    }
    if (values) {
      const bf16x8* src = a.VA + b * a.va_user_frags + static_cast<int64_t>(head) * K3 * MB * 64;
#pragma unroll
      for (int kk = 0; kk < K3; ++kk)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) va[kk][mb] = src[(kk * MB + mb) * 64 + lane];
    }
  };
  // item t of the first user's operands, in the order of their first use (the keys, then the values)
  constexpr int nKA = FUSED ? 0 : K2 * LB, nVA = WEIGHTS ? 0 : K3 * MB, nUser = nKA + nVA;
  auto load_user_item = [&](int b, int t) {
    if (t < nKA) {
      const bf16x8* src = a.KA + b * a.ka_user_frags + static_cast<int64_t>(head) * K2 * LB * 64;
      ka[t / LB][t % LB] = src[t * 64 + lane];
    } else {
      const int u = t - nKA;
      const bf16x8* src = a.VA + b * a.va_user_frags + static_cast<int64_t>(head) * K3 * MB * 64;
      va[u / MB][u % MB] = src[u * 64 + lane];
    }
  };
  int cur_user = first / a.tiles_per_user;
  if constexpr (!kJit) load_user(cur_user, !FUSED, !WEIGHTS);  // requested with everything else, long before their first use
  int rlen = a.row_lens ? min(a.row_lens[cur_user], a.rows) : a.rows;

  // Software pipeline: while the vector ALUs do phi of tile i, the matrix cores already run the
  // first product of tile i+1, whose X rows were parked in the other LDS buffer.
  park(ring[0], xs[0]);
  __syncthreads();
  if constexpr (kJit) {
    first_begin(xs[0]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) {
      if (kk + kLead < KR) {
        load_wq_step(kk + kLead);
      } else {
        const int slot = kk + kLead - KR;  // 0 .. kLead - 1: the k-steps that have no W_Q^T left to ask for
#pragma unroll
        for (int t = slot * nUser / kLead; t < (slot + 1) * nUser / kLead; ++t) load_user_item(cur_user, t);
      }
#pragma unroll
      for (int mb = 0; mb < FB; ++mb) first_mfma(kk * FB + mb);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (first + P < last) {
      issue(ib, ir0, ring[0]);
      advance(ib, ir0);
    }
  } else {
    if (first + P < last) {
      issue(ib, ir0, ring[0]);
      advance(ib, ir0);
    }
    first_product(xs[0]);
  }
  int b = b_first, r0 = r0_first;  // the tile being computed

  for (int base = first; base < last; base += P) {
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int tile = base + p;
      if (tile >= last) break;  // uniform over the workgroup
      const bool has_next = tile + 1 < last;
      if (b != cur_user) {
        // A new user's operands are waited for right here, inside the rare branch: left pending, they
        // would make every tile wait for all of its outstanding loads and stores before the second product.
        load_user(b, !FUSED && a.ka_user_frags != 0, !WEIGHTS && a.va_user_frags != 0);
        rlen = a.row_lens ? min(a.row_lens[b], a.rows) : a.rows;
        cur_user = b;
#pragma unroll
        for (int kk = 0; kk < K2; ++kk)
#pragma unroll
          for (int lb = 0; lb < LB; ++lb) asm volatile("" : "+v"(ka[kk][lb]));
#pragma unroll
        for (int kk = 0; kk < K3; ++kk)
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) asm volatile("" : "+v"(va[kk][mb]));
        asm volatile("" : "+v"(rlen));
      }

      if constexpr (FUSED) {
        // the first product already is S^T; the next tile's accumulates in the other set of registers
#pragma unroll
        for (int lb = 0; lb < LB; ++lb) acc2[lb] = acc1[lb];
      } else {
        // S^T = K~_a Q~^T from this tile's first product
        bf16x8 qf[K2];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          qf[2 * mb] = pack_half(acc1[mb], 0);
          qf[2 * mb + 1] = pack_half(acc1[mb], 1);
        }
        // (the link blocks' chains interleaved: products into one accumulator issue every 51 cycles, into two in
        // turn every 37)
#pragma unroll
        for (int lb = 0; lb < LB; ++lb)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc2[lb][i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < K2; ++kk)
#pragma unroll
          for (int lb = 0; lb < LB; ++lb) acc2[lb] = mfma32(ka[kk][lb], qf[kk], acc2[lb]);
      }

      float inv;
      if (has_next) {
        // The buffer being overwritten was last read for the tile before this one; every wave has
        // passed a barrier since.  The barrier below publishes the new tile.
        unsigned char* nbuf = xs[(p + 1) & 1];
        park(ring[(p + 1) % P], nbuf);
        __syncthreads();
        if (tile + P + 1 < last) {
          issue(ib, ir0, ring[(p + 1) % P]);
          advance(ib, ir0);
        }
        // one MFMA of the next tile's first product, then its share of phi's steps, and so on; the
        // fences keep the compiler from regrouping them
        first_begin(nbuf);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NM; ++i) {
          first_mfma(i);
#pragma unroll
          for (int st = i * NV / NM; st < (i + 1) * NV / NM; ++st) phi_step(st);
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int st = 0; st < NV; ++st) phi_step(st);
      }
      inv = phi_finish();
      if constexpr (WEIGHTS) {
        // register 4j + r of block lb is link 32 lb + 8 j + 4 g + r of this lane's query row
        const int row = r0 + n;
        if (row < a.rows) {
          bf16_t* wrow = a.Wout + ((static_cast<int64_t>(b) * a.rows + row) * H + head) * M + 4 * g;
#pragma unroll
          for (int lb = 0; lb < LB; ++lb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              bf16x4 v;
#pragma unroll
              for (int r = 0; r < 4; ++r) v[r] = static_cast<__bf16>(acc2[lb][4 * j + r] * inv);
              *reinterpret_cast<bf16x4*>(wrow + 32 * lb + 8 * j) = v;
            }
        }
      } else {
      // O^T = V~_a^T phi(S)^T; lane (n, g) gets 16 consecutive columns per block.  The wave's 32 x d/h
      // output tile goes through LDS so that whole 2*d/h-byte row segments are stored at once.
      unsigned char* otile = os[head];
      f32x16 acc3[MB];
#pragma unroll
      for (int ob = 0; ob < MB; ++ob)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc3[ob][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K3; ++kk)
#pragma unroll
        for (int ob = 0; ob < MB; ++ob) acc3[ob] = mfma32(va[kk][ob], pf[kk], acc3[ob]);
#pragma unroll
      for (int ob = 0; ob < MB; ++ob) {
        bf16x8 lo, hi;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          lo[t] = static_cast<__bf16>(acc3[ob][t] * inv);
          hi[t] = static_cast<__bf16>(acc3[ob][8 + t] * inv);
        }
        unsigned char* dst = otile + n * OPITCH + (32 * ob + 16 * g) * 2;
        *reinterpret_cast<bf16x8*>(dst) = lo;
        *reinterpret_cast<bf16x8*>(dst + 16) = hi;
      }
      // all reads of the staged tile first, then the stores: one LDS round trip instead of LW
      bf16x8 ov[LW];
#pragma unroll
      for (int j = 0; j < LW; ++j) {
        const int q = j * 64 + lane;
        ov[j] = *reinterpret_cast<const bf16x8*>(otile + (q / OCPR) * OPITCH + (q % OCPR) * 16);
      }
      __builtin_amdgcn_sched_barrier(0);
      unsigned char* obase = reinterpret_cast<unsigned char*>(a.O) +
                             ((static_cast<int64_t>(b) * a.rows + r0) * D + head * DH) * 2;
      if (r0 + 32 <= min(rlen, a.rows)) {  // uniform: every row of the tile is stored as computed
#pragma unroll
        for (int j = 0; j < LW; ++j) store_through(obase, 32 * 2 * D, ooff[j], ov[j]);
      } else {
#pragma unroll
        for (int j = 0; j < LW; ++j) {
          const int row = r0 + (j * 64 + lane) / OCPR;
          bf16x8 v = ov[j];
          if (row >= rlen) {
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = static_cast<__bf16>(0.f);
          }
          if (row < a.rows) *reinterpret_cast<bf16x8*>(obase + ooff[j]) = v;
        }
      }
      }
      advance(b, r0);
    }
  }
}


template <int DH, int M, int H, bool FUSED>
hipError_t launch_form(const MainArgs& m, int phi, int grid, hipStream_t s) {
  if (m.Wout != nullptr)
    launch_timed(kKernelQueriesOverLinks, queries_over_links_kernel<DH, M, H, kPhiSoftmax, true, FUSED>, dim3(grid), dim3(64 * H), 0, s, m);
  else if (phi == kPhiSoftmax && m.ln_on) {
    if constexpr (FUSED) return hipErrorInvalidValue;
    else launch_timed(kKernelQueriesOverLinks, queries_over_links_kernel<DH, M, H, kPhiSoftmax, false, false, true>, dim3(grid), dim3(64 * H), 0, s, m);
  } else if (m.ln_on)
    return hipErrorInvalidValue;
  else if (phi == kPhiSoftmax)
    launch_timed(kKernelQueriesOverLinks, queries_over_links_kernel<DH, M, H, kPhiSoftmax, false, FUSED>, dim3(grid), dim3(64 * H), 0, s, m);
  else
    launch_timed(kKernelQueriesOverLinks, queries_over_links_kernel<DH, M, H, kPhiSilu, false, FUSED>, dim3(grid), dim3(64 * H), 0, s, m);
  return hipGetLastError();
}

template <int DH, int M, int H>
hipError_t launch_main(const MainArgs& m, int phi, int grid, hipStream_t s) {
  if (m.fused) {
    if constexpr (M <= DH) return launch_form<DH, M, H, true>(m, phi, grid, s);
    return hipErrorInvalidValue;
  }
  return launch_form<DH, M, H, false>(m, phi, grid, s);
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

// One contraction X G instead of X W_Q followed by the product with K~: possible when the keys are shared, and
// no more work or registers when there are at most as many links as head columns.
bool fused_scores(int d, int h, int m, bool k_per_user) { return !k_per_user && m <= d / h; }

size_t queries_over_links_workspace(int B, int d, int m, bool k_per_user) {
  const size_t wq = align_up(static_cast<size_t>(d) * d * 2 + kQueryImagePadBytes);
  const size_t ka = align_up(static_cast<size_t>(k_per_user ? B : 1) * m * d * 2);
  const size_t va = align_up(static_cast<size_t>(B) * m * d * 2);
  return wq + ka + va;
}

void* queries_over_links_values(const QueriesOverLinks& q, void* workspace) {
  char* ws = static_cast<char*>(workspace);
  return ws + align_up(static_cast<size_t>(q.d) * q.d * 2 + kQueryImagePadBytes) +
         align_up(static_cast<size_t>(q.k_user_stride != 0 ? q.B : 1) * q.m * q.d * 2);
}

void queries_over_links_jobs(const QueriesOverLinks& q, void* workspace, PackJobs& jobs, bool values) {
  const int d = q.d, m = q.m;
  const bool k_per_user = q.k_user_stride != 0, v_per_user = q.v_user_stride != 0;
  char* ws = static_cast<char*>(workspace);
  char* KA = ws + align_up(static_cast<size_t>(d) * d * 2 + kQueryImagePadBytes);
  char* VA = KA + align_up(static_cast<size_t>(k_per_user ? q.B : 1) * m * d * 2);
  jobs.weights[jobs.n_weights++] = PackWeight{q.Wq, ws, 1.f, kQueryImageHeadPad};
  // a negative logit scale is folded into the sign of the packed keys, so the kernel sees scale >= 0
  jobs.projections[jobs.n_projections++] =
      PackProject{q.Ksrc, q.Wk, KA, q.k_user_stride, k_per_user ? q.B : 1, kPackKeys, q.scale < 0.f ? -1.f : 1.f, q.k_norm};
  if (!q.weights_out && values)
    jobs.projections[jobs.n_projections++] = PackProject{q.Vsrc, q.Wv, VA, q.v_user_stride, v_per_user ? q.B : 1, kPackValues, 1.f, q.v_norm};
}

hipError_t queries_over_links(const QueriesOverLinks& q, void* workspace, hipStream_t s) {
  const int d = q.d, h = q.h, m = q.m, dh = d / h;
  const bool k_per_user = q.k_user_stride != 0, v_per_user = q.v_user_stride != 0;
  char* ws = static_cast<char*>(workspace);
  bf16_t* WqA = reinterpret_cast<bf16_t*>(ws);
  bf16_t* KA = reinterpret_cast<bf16_t*>(ws + align_up(static_cast<size_t>(d) * d * 2 + kQueryImagePadBytes));
  bf16_t* VA = reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(KA) +
                                         align_up(static_cast<size_t>(k_per_user ? q.B : 1) * m * d * 2));
  // The score image G costs more to build than W_Q^T and K~ do to pack (measured twice: 0.7 us off this kernel against
  // 3 us more for the request when it is built per call), so it replaces them only where it is built once per model.
  const bool fused = q.prepared != nullptr && fused_scores(d, h, m, k_per_user);
  hipError_t e = hipSuccess;
  if (q.prepared != nullptr) {  // only the user's values are left to pack
    const PreparedLayout l = prepared_layout(d, m);
    WqA = reinterpret_cast<bf16_t*>(const_cast<char*>(static_cast<const char*>(q.prepared)) + l.wq);
    KA = reinterpret_cast<bf16_t*>(const_cast<char*>(static_cast<const char*>(q.prepared)) + l.ka);
    PackProject vjob{q.Vsrc, q.Wv, VA, q.v_user_stride, v_per_user ? q.B : 1, kPackValues, 1.f};
    if (!q.packed) e = pack_operands(nullptr, 0, &vjob, q.weights_out ? 0 : 1, d, h, m, s);
  } else if (!q.packed) {
    PackJobs jobs;
    queries_over_links_jobs(q, workspace, jobs);
    e = pack_operands(jobs, d, h, m, s);
  }
  if (e != hipSuccess) return e;

  MainArgs a{};
  a.X = static_cast<const bf16_t*>(q.X), a.O = static_cast<bf16_t*>(q.O);
  a.WqA = reinterpret_cast<const bf16x8*>(WqA), a.KA = reinterpret_cast<const bf16x8*>(KA);
  a.VA = reinterpret_cast<const bf16x8*>(VA);
  a.ka_user_frags = k_per_user ? static_cast<int64_t>(m) * d / 8 : 0;
  a.va_user_frags = v_per_user ? static_cast<int64_t>(m) * d / 8 : 0;
  a.row_lens = q.row_lens;
  a.Wout = static_cast<bf16_t*>(q.weights_out);
  a.fused = fused;
  a.ln_on = q.x_norm.on, a.ln_eps = q.x_norm.eps;
  a.ln_gamma = static_cast<const bf16_t*>(q.x_norm.gamma), a.ln_beta = static_cast<const bf16_t*>(q.x_norm.beta);
  a.B = q.B, a.rows = q.rows, a.tiles_per_user = (q.rows + 31) / 32;
  a.total_tiles = a.tiles_per_user * q.B;  // the caller has checked that this fits an int
  a.scale = fabsf(q.scale), a.inv_norm = 1.f / static_cast<float>(m);
  // one resident workgroup per compute unit when the kernel needs most of the register file,
  // two when its footprint is small (d/h = 32)
  const int resident = compute_units() * (dh == 32 && h <= 4 ? 2 : 1);
  const int grid = a.total_tiles < resident ? a.total_tiles : resident;
  e = dh == 32 ? dispatch_h<32>(a, h, m, q.phi, grid, s) : dispatch_h<64>(a, h, m, q.phi, grid, s);
  return e;
}

}  // namespace lime
