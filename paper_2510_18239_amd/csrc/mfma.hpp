// bf16 matrix-core (MFMA) building blocks for gfx950 and the launcher interface of the
// kernels built from them.
//
// All contractions use v_mfma_f32_32x32x16_bf16.  With lane = 32*g + n (n in [0,32), g in {0,1}):
//   A fragment (32 x 16):  lane holds A[row n][k = 8g + t], t = 0..7
//   B fragment (16 x 32):  lane holds B[k = 8g + t][col n]
//   D accumulator (32x32): lane holds D[row 8j + 4g + r][col n] in register 4j + r (j, r in [0,4))
// The two operand layouts are mirror images (lane <-> the index that is kept, slot <-> the index
// that is summed), so a D block can be fed straight back as an operand whose summed index is D's
// row index: registers 8f..8f+7 (f in {0,1}) of a D block form one 16-deep fragment in which slot t
// of lane-half g stands for row 16f + chain_k(g, t).  The other operand of that product is laid
// out in the same "chained" order; sums do not care about the order of their terms.
#pragma once

#include "common.hpp"

namespace lime {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row (within a 16-deep k-step) that slot t of lane-half g stands for in a chained fragment.
__host__ __device__ constexpr int chain_k(int g, int t) { return 8 * (t >> 2) + 4 * g + (t & 3); }
// Inverse: k in [0,16) -> lane-half and slot.
__host__ __device__ constexpr int chain_g(int k) { return (k >> 2) & 1; }
__host__ __device__ constexpr int chain_t(int k) { return 4 * (k >> 3) + (k & 3); }

// Registers 8f..8f+7 of a D block as a bf16 fragment (round to nearest even).
__device__ __forceinline__ bf16x8 pack_half(const f32x16& d, int f) {
  bf16x8 r;
#pragma unroll
  for (int t = 0; t < 8; ++t) r[t] = static_cast<__bf16>(d[8 * f + t]);
  return r;
}

// Reductions over the lane pair (n, n + 32), which together hold one row of an accumulator block.
// v_permlane32_swap exchanges the wave's halves in the vector ALU (no LDS round trip): with both operands x it
// returns (x of the low half, x of the high half) in every lane, so both lanes of a pair compute the same bits.
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float pair_max(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Sums over groups of G neighbouring lanes (G a power of two, groups aligned), every lane of a group getting the
// group's sum, without an LDS round trip where G is 16 or 32: four DPP rotations inside the 16-lane row, then
// v_permlane16_swap, which with both operands x returns (x of the even row, x of the odd row) of the lane's row pair.
template <int N>
__device__ __forceinline__ float row_rotated(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 + N, 0xF, 0xF, false));  // row_ror:N
}
template <int G>
__device__ __forceinline__ float group_sum(float x) {
  if constexpr (G == 16 || G == 32) {
    x += row_rotated<8>(x);
    x += row_rotated<4>(x);
    x += row_rotated<2>(x);
    x += row_rotated<1>(x);
    if constexpr (G == 32) {
      const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
      x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
  } else {
#pragma unroll
    for (int o = 1; o < G; o *= 2) x += __shfl_xor(x, o, 64);
  }
  return x;
}

__device__ __forceinline__ float wave_sum(float x) { return pair_sum(group_sum<32>(x)); }

// A 16-byte store that writes through the L2 (agent scope, `sc1`): `base` is uniform over the wave, `offset` the
// lane's byte offset below `span` bytes.  The XCDs' L2s are not coherent with each other, so whatever a kernel
// leaves dirty in them is written back when the kernel ends; an output stream that nobody on the chip reads again is
// better written through as it is produced (measured on the candidate-side kernel at 32 768 rows: 14.9 -> 13.7 us).
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_through(void* base, int span, int offset, bf16x8 v) {
  const auto rsrc = __builtin_amdgcn_make_buffer_rsrc(base, 0, span, 0x00020000);
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rsrc, offset, 0, 16 /* sc1 */);
}

// Output-row permutation that makes a lane's 16 accumulator registers 16 consecutive columns:
// the A-operand row `rho` of an output block carries column out_col(rho); lane-half g then holds
// columns 16g .. 16g+15 of the 32-wide block in register order.
__host__ __device__ constexpr int out_col(int rho) { return 16 * ((rho >> 2) & 1) + 4 * (rho >> 3) + (rho & 3); }
__host__ __device__ constexpr int out_rho(int col) { return 8 * ((col >> 2) & 3) + 4 * (col >> 4) + (col & 3); }

// ----------------------------------------------------------------------------- operand packing (mfma_pack.hip)
// One small kernel per call lays the stationary operands out in fragment order (units of bf16x8,
// one per lane), so that the main kernels fetch each fragment with one 16-byte access per lane.
//   weight image  [h][d/16][dh/32][64]: fragment (a, kk, mb), lane (n, g), slot t = W[16kk + 8g + t][a dh + 32mb + n]
//     (the head-a slice of W^T as an A operand with natural k order; equally W as a B operand)
//   kPackKeys     [U][h][dh/16][m/32][64]: fragment (u, a, kk, lb), lane (n, g), slot t
//                   = (X_u W)[32lb + n][a dh + 16kk + chain_k(g, t)]   (rows kept, head columns summed in chained order)
//   kPackValues   [U][h][m/16][dh/32][64]: fragment (u, a, kk, ob), lane (rho, g), slot t
//                   = (X_u W)[16kk + chain_k(g, t)][a dh + 32ob + out_col(rho)]   (rows summed in chained order)
// Where element (row, col) of a projected [m][d] matrix goes in its fragment image (bf16 units).
__device__ __forceinline__ int64_t keys_slot(int u, int row, int col, int d, int dh, int m) {
  const int a = col / dh, c = col % dh, kk = c / 16, kin = c % 16;
  const int64_t frag = ((static_cast<int64_t>(u) * (d / dh) + a) * (dh / 16) + kk) * (m / 32) + row / 32;
  return (frag * 64 + 32 * chain_g(kin) + row % 32) * 8 + chain_t(kin);
}
__device__ __forceinline__ int64_t values_slot(int u, int row, int col, int d, int dh, int m, bool chained) {
  const int a = col / dh, c = col % dh, kk = row / 16, kin = row % 16;
  const int64_t frag = ((static_cast<int64_t>(u) * (d / dh) + a) * (m / 16) + kk) * (dh / 32) + c / 32;
  const int g = chained ? chain_g(kin) : kin / 8, t = chained ? chain_t(kin) : kin % 8;
  return (frag * 64 + 32 * g + out_rho(c % 32)) * 8 + t;
}

// Fragments (1 KiB each) left free between the head slices of the candidate side's query-weight image (and of the
// score image that replaces it).  Zero: starting the heads' slices at different cache-channel phases was measured
// and changed nothing.
constexpr int kQueryImageHeadPad = 0;
constexpr size_t kQueryImagePadBytes = 8 * 1024 * static_cast<size_t>(kQueryImageHeadPad);  // up to eight heads
struct PackWeight {
  const void* W;   // [d][d] bf16, or nullptr for the identity
  void* image;
  float sign = 1.f;  // +1 or -1, multiplies every element (exact)
  int head_pad = 0;  // fragments left free between the head slices of the image
};
// Layer normalisation of an operand's rows on their way into a kernel (Appendix C: the tensors that enter an MHA are
// normalised before the Q, K, V projections): y = (x - mean) / sqrt(var + eps) * gamma + beta over the d features
// (biased variance, statistics in fp32, mean first and then the centred second moment), rounded to bf16 exactly
// where a separate normalisation pass would have stored it.  gamma, beta [d] bf16, both required when `on` (the
// kernels fetch them unconditionally, together with their other operands).
struct RowNorm {
  bool on = false;
  const void* gamma = nullptr;
  const void* beta = nullptr;
  float eps = 0.f;
};
//   kPackValuesNatural: as kPackValues with the rows summed in natural order, 16kk + 8g + t (for a B operand
//                   that is read row-major from memory rather than taken from accumulators)
constexpr int kPackKeys = 0, kPackValues = 1, kPackValuesNatural = 2;
struct PackProject {
  const void* X;   // [users][m][d] bf16 rows to project
  const void* W;   // [d][d] bf16, or nullptr for the identity
  void* image;
  int64_t user_stride;  // elements between users in X
  int users;
  int layout;      // kPackKeys, kPackValues or kPackValuesNatural
  float sign;      // +1 or -1: multiplies every projected element (exact); lets kernels assume scale >= 0
  RowNorm norm;    // applied to the rows of X before the projection
};
//   score image   [h][d/16][m/32][64]: fragment (a, kk, lb), lane (n, g), slot t = G_a[16kk + 8g + t][32lb + n] with
//                   G_a = W_Q[:, head a] (L W_K)[:, head a]^T  (d x m): the logits of head a are X G_a, so when the keys
//                   do not depend on the user (Section 3.3) the query projection and the key product collapse into one
//                   contraction over d.  Same shape as a weight image with the m links in place of the head's columns.
struct PackScore {
  const void* Wq;    // [d][d] bf16, or nullptr for the identity
  const void* Ksrc;  // [m][d] bf16 rows that become keys (shared by all users)
  const void* Wk;    // [d][d] bf16, or nullptr for the identity
  void* image;
  float sign;        // +1 or -1
};
constexpr int kMaxPackWeights = 8, kMaxPackProjections = 3;  // jobs one launch takes
hipError_t pack_operands(const PackWeight* weights, int n_weights, const PackProject* projections, int n_projections,
                         int d, int h, int m, hipStream_t s, const PackScore* score = nullptr);
// Jobs collected from several users of the pack kernel (same d, h, m), to be written by one launch.
struct PackJobs {
  PackWeight weights[kMaxPackWeights];
  int n_weights = 0;
  PackProject projections[kMaxPackProjections];
  int n_projections = 0;
  PackScore score{};      // at most one score image per launch
  bool has_score = false;
};
hipError_t pack_operands(const PackJobs& jobs, int d, int h, int m, hipStream_t s);

// ----------------------------------------------------------------------------- operands prepared once per model
// What the two stages need of the model alone -- weights and shared links, not the user -- packed once into a
// caller-owned buffer: for the history stage the W_K^T and W_V images and the projected link queries
// Q~ = L^C W_Q; for the candidate stage the W_Q^T image and the projected link keys K~ = L W_K.  The signs of
// the two logit scales are folded in.  The stages then skip their own packing of these.
struct PreparedLayout {
  size_t wk, wv, qb, wq, ka, total;  // byte offsets of the five images, and the size of the buffer
};
PreparedLayout prepared_layout(int d, int m);
struct PrepareOperands {
  const void* LC;   // [m][d] shared contextualised links (history-stage queries)
  const void* L;    // [m][d] raw links (candidate-stage keys)
  const void *Wq_hist, *Wk_hist, *Wv_hist;  // history-stage weights, all required
  const void *Wq_cand, *Wk_cand;            // candidate-stage weights, nullable = identity
  float scale_hist, scale_cand;
  int d, h, m;
};
hipError_t prepare_operands(const PrepareOperands& p, void* prepared, hipStream_t s);

// ----------------------------------------------------------------------------- candidate-side kernel family
// Fused "queries x few keys" attention: for every query row x (a candidate of Eq. 4, or a history
// row for O[S] of Eq. 7): q = x Wq; per head w = phi(scale * q K~^T) over the m keys; out = w V~.
struct QueriesOverLinks {
  const void* X;        // [B][rows][d] bf16 query-side embeddings (T, or E for O[S])
  void* O;              // [B][rows][d] bf16
  const void* Wq;       // [d][d] bf16 or nullptr (identity)
  const void* Ksrc;     // [.][m][d] bf16 rows that become keys   (L, or LC)
  const void* Wk;       // nullable
  const void* Vsrc;     // [.][m][d] bf16 rows that become values (LP, or LC)
  const void* Wv;       // nullable
  int64_t k_user_stride, v_user_stride;  // elements; 0 = shared
  const int32_t* row_lens;               // nullable; rows >= row_lens[b] are written as zeros
  int B, rows, d, h, m;
  float scale;
  int phi;              // kPhiSoftmax, or kPhiSilu with normaliser m
  void* weights_out;    // when set: write the attention weights [B][rows][h][m] instead of O (Vsrc, Wv unused)
  const void* prepared; // when set: W_Q^T and K~ come from this prepared buffer (Wq, Ksrc, Wk unused; shared keys)
  bool packed;          // when set: the operands have been packed into the workspace already (queries_over_links_jobs;
                        // with `prepared`: the value image, by the history side's merge step)
  RowNorm x_norm;       // applied to the query rows as their tiles are loaded (softmax, O output, per-call operands)
  RowNorm k_norm, v_norm;  // applied to the key / value rows by the pack step
};
// where the value image of a call lives in its workspace
void* queries_over_links_values(const QueriesOverLinks& a, void* workspace);
// The pack jobs of a call, appended to `jobs` instead of being launched by queries_over_links (not with `prepared`);
// without `values` when someone else writes the value image (the history side's merge step).
void queries_over_links_jobs(const QueriesOverLinks& a, void* workspace, PackJobs& jobs, bool values = true);
bool queries_over_links_supported(int d, int h, int m);
bool fused_scores(int d, int h, int m, bool k_per_user);  // whether the kernel takes the score image G
size_t queries_over_links_workspace(int B, int d, int m, bool k_per_user);
hipError_t queries_over_links(const QueriesOverLinks& a, void* workspace, hipStream_t s);

// ----------------------------------------------------------------------------- QK-cache scoring (mfma_cached.hip)
struct CachedCandidates {
  const void* W;    // [B][C][h][m] bf16 cached attention weights; with ids: the table [n_items][h][m]
  const int32_t* ids;  // nullable: [B][C] rows of the table; an id outside [0, n_items) gives a zero output row
  int n_items;
  const void* LP;   // [B][m][d] bf16
  const void* Wv;   // nullable
  void* O;          // [B][C][d] bf16
  int B, C, d, h, m;
};
size_t cached_candidates_workspace(int B, int d, int m);
hipError_t cached_candidates(const CachedCandidates& a, void* workspace, hipStream_t s);

// ----------------------------------------------------------------------------- baseline: full target attention
struct TargetAttention {
  const void* T;        // [B][C][d] bf16
  const void* E;        // [B][N][d] bf16
  const int32_t* lens;  // nullable
  const void *Wq, *Wk, *Wv;
  void* O;              // [B][C][d] bf16
  int B, C, N, d, h;
  float scale;
};
bool target_attention_supported(int d, int h);
size_t target_attention_workspace(int B, int C, int N, int d);
hipError_t target_attention(const TargetAttention& a, void* workspace, hipStream_t s);

// ----------------------------------------------------------------------------- gated block of an XOR layer (mfma_layers.hip)
// The gated block of an XOR layer in one kernel: Y = X + (A * SiLU(X Wu)) Wo per row (rows >= lens[b] are zeros), and
// optionally sum_out / sum_rounded = sum_in + (A * SiLU(X Wu)) Wo (the running sum of the layers' link outputs).
struct GatedBlock {
  const void* X;          // [.][rows][d] bf16
  int64_t x_user_stride;  // elements between users; 0 = one [rows][d] block for all users
  const int32_t* lens;    // nullable
  const void *Wu_image, *Wo_image;  // weight images written by pack_operands
  const void* A;          // [B][rows][d] bf16
  void* Y;                // [B][rows][d] bf16, nullable
  const float* sum_in;    // nullable = zero
  float* sum_out;         // nullable
  void* sum_rounded;      // bf16, nullable
  int B, rows, d, h;
};
hipError_t gated_block(const GatedBlock& q, hipStream_t s);

// ----------------------------------------------------------------------------- history-side kernel family
// Fused "few queries x many keys" attention: the m links attend over one user's N history rows;
// keys and values are projected on the fly (K~ = E Wk, V~ = E Wv), queries are Q~ = LC Wq.
struct LinksOverHistory {
  const void* E;        // [B][N][d] bf16
  const int32_t* lens;  // nullable
  const void* LC;       // [.][m][d] bf16
  int64_t lc_user_stride;
  const void *Wq, *Wk, *Wv;  // [d][d] bf16, all required
  void* LP;             // [B][m][d] bf16
  int B, N, d, h, m;
  float scale;
  int phi;              // kPhiSoftmax, or kPhiSilu with normaliser lens[b]
  const void* prepared; // when set: W_K^T, W_V and Q~ come from this prepared buffer (LC, Wq, Wk, Wv unused)
  bool packed;          // when set: the operands have been packed into the workspace already (links_over_history_jobs)
  // when values_image is set, the merge step also projects the link states it has just finished, V~ = LP Wv_values
  // (Wv_values [d][d] bf16, nullable = identity), and writes them as the kPackValues image of a candidate-side call
  const void* Wv_values;
  void* values_image;
  RowNorm values_norm;  // applied to the finished link states before that projection (LP itself is stored as it is)
  RowNorm q_norm;       // applied to the link rows LC by the pack step
};
void links_over_history_jobs(const LinksOverHistory& a, void* workspace, PackJobs& jobs);
bool links_over_history_supported(int d, int h, int m);
size_t links_over_history_workspace(int B, int N, int d, int h, int m, bool q_per_user);
hipError_t links_over_history(const LinksOverHistory& a, void* workspace, hipStream_t s);

}  // namespace lime
