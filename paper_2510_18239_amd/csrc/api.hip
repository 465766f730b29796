// C ABI of the LIME hot path: argument checks, workspace planning, kernel dispatch.
#include "../../include/lime.h"

#include <stdarg.h>
#include <stdio.h>

#include <algorithm>
#include <mutex>

#include "common.hpp"
#include "mfma.hpp"
#include "scoring.hpp"

// Scratch of lime_request_static, the entry point for callers that cannot allocate or pass a workspace: 16 MiB per
// GPU, held from the moment the library's code is loaded on that GPU until the process ends.
constexpr size_t kStaticScratchBytes = size_t{16} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_error[512] = "";

int32_t fail(int32_t status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return status;
}

}  // namespace

namespace lime {
int32_t set_error(int32_t status, const char* text) { return fail(status, "%s", text); }
}  // namespace lime

namespace {

#define LIME_HIP(expr)                                                                            \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return fail(LIME_LAUNCH_FAILED, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

constexpr int kMaxHeadDim = 256;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
template <typename... P>
bool all_aligned16(P... p) { return (aligned16(p) && ...); }
// the matrix-core kernels index 32-row tiles with an int
bool fits_tiles(int64_t users, int64_t rows) { return users * ((rows + 31) / 32) < (int64_t{1} << 31); }
constexpr int kMaxUsers = 65535;

// Carves 256-byte aligned pieces out of the caller's workspace; with base == nullptr it only sizes.
struct Arena {
  char* base;
  size_t used = 0;
  explicit Arena(void* p) : base(static_cast<char*>(p)) {}
  template <typename T>
  T* take(size_t count) {
    T* p = base ? reinterpret_cast<T*>(base + used) : nullptr;
    used += lime::align_up(count * sizeof(T));
    return p;
  }
};

int32_t check_common(const char* fn, int32_t B, int32_t d, int32_t h, int32_t dtype) {
  if (dtype != LIME_F32 && dtype != LIME_BF16) return fail(LIME_INVALID_ARG, "%s: unknown dtype %d", fn, dtype);
  if (B <= 0 || d <= 0 || h <= 0) return fail(LIME_INVALID_ARG, "%s: B, d, h must be positive (B=%d d=%d h=%d)", fn, B, d, h);
  if (d % h != 0) return fail(LIME_INVALID_ARG, "%s: d=%d is not a multiple of h=%d", fn, d, h);
  if (d / h > kMaxHeadDim) return fail(LIME_UNSUPPORTED, "%s: d/h=%d exceeds %d", fn, d / h, kMaxHeadDim);
  if (B > kMaxUsers) return fail(LIME_UNSUPPORTED, "%s: B=%d exceeds %d", fn, B, kMaxUsers);
  return LIME_OK;
}

// ----------------------------------------------------------------------------- history side (Eq. 3, Eq. 7)
struct HistoryPlan {
  float *Qt, *Ks, *Vs;        // Q[T] = LC Wq; K[S] = E Wk; V[S] = E Wv
  float *Qs, *Kt, *Vt;        // only for O[S]: Q[S] = E Wq; K[T] = LC Wk; V[T] = LC Wv
  size_t bytes;
};

HistoryPlan plan_history(void* ws, int64_t B, int64_t N, int64_t d, int64_t m, bool per_user_links, bool want_os) {
  Arena a(ws);
  HistoryPlan p{};
  const int64_t link_rows = (per_user_links ? B : 1) * m;
  p.Qt = a.take<float>(link_rows * d);
  p.Ks = a.take<float>(B * N * d);
  p.Vs = a.take<float>(B * N * d);
  if (want_os) {
    p.Qs = a.take<float>(B * N * d);
    p.Kt = a.take<float>(link_rows * d);
    p.Vt = a.take<float>(link_rows * d);
  }
  p.bytes = a.used;
  return p;
}

// Workspace of lime_xor_layers: one XORA layer's own workspace, the tensors that travel between the steps of a layer
// (storage type) and the running sum of the link outputs (fp32); on the matrix cores also the two weight images of
// the current layer, on the general kernels the scratch of the gated block.
struct XorLayersPlan {
  void* hist_ws;
  size_t hist_bytes;
  void *Wu_image, *Wo_image;
  void *Xs[2], *OS;        // history rows [B][N][d]: the residual stream (two copies, alternating) and O[S]
  void *Xt[2], *OT;        // link rows [B][m][d]: the same three
  float* sum;              // [B][m][d]
  float* P;                // general kernels: [B][max(N, m)][d] fp32 ...
  void* Z;                 // ... and the same in the storage type
  size_t bytes;
};

XorLayersPlan plan_xor_layers(void* ws, int64_t B, int64_t N, int64_t d, int64_t h, int64_t m, int32_t dtype, bool on_mfma) {
  Arena a(ws);
  XorLayersPlan p{};
  const size_t es = dtype == LIME_BF16 ? 2 : 4;
  // (sized for whichever kernels the XORA step picks: with misaligned caller tensors the first layer runs on the
  // general kernels and the later ones, whose inputs live in this workspace, on the matrix cores)
  p.hist_bytes = plan_history(nullptr, B, N, d, m, true, true).bytes;
  if (dtype == LIME_BF16 && lime::links_over_history_supported(d, h, m))
    p.hist_bytes = std::max(p.hist_bytes, lime::links_over_history_workspace(B, N, d, h, m, true) +
                                              lime::queries_over_links_workspace(B, d, m, true));
  p.hist_ws = a.take<char>(p.hist_bytes);
  if (on_mfma) {
    p.Wu_image = a.take<uint16_t>(d * d);
    p.Wo_image = a.take<uint16_t>(d * d);
  } else {
    p.P = a.take<float>(B * std::max(N, m) * d);
    p.Z = a.take<char>(B * std::max(N, m) * d * es);
  }
  for (void** t : {&p.Xs[0], &p.Xs[1], &p.OS}) *t = a.take<char>(B * N * d * es);
  for (void** t : {&p.Xt[0], &p.Xt[1], &p.OT}) *t = a.take<char>(B * m * d * es);
  p.sum = a.take<float>(B * m * d);
  p.bytes = a.used;
  return p;
}

// large enough for either path (a bf16 call whose pointers are not 16-byte aligned runs on the general kernels)
size_t xor_layers_workspace(int64_t B, int64_t N, int64_t d, int64_t h, int64_t m, int32_t dtype) {
  size_t need = plan_xor_layers(nullptr, B, N, d, h, m, dtype, false).bytes;
  if (dtype == LIME_BF16 && lime::links_over_history_supported(d, h, m))
    need = std::max(need, plan_xor_layers(nullptr, B, N, d, h, m, dtype, true).bytes);
  return need;
}

// O[S] of XORA on the candidate-side kernel: every history row attends over the m links, SiLU / m.
lime::QueriesOverLinks os_query(const void* E, const int32_t* lens, const void* LC, int64_t link_stride, const void* Wq,
                                const void* Wk, const void* Wv, void* OS, int32_t B, int32_t N, int32_t d, int32_t h,
                                int32_t m, float scale) {
  lime::QueriesOverLinks q{};
  q.X = E, q.O = OS, q.Wq = Wq, q.Ksrc = LC, q.Wk = Wk, q.Vsrc = LC, q.Wv = Wv;
  q.k_user_stride = q.v_user_stride = link_stride, q.row_lens = lens;
  q.B = B, q.rows = N, q.d = d, q.h = h, q.m = m, q.scale = scale, q.phi = lime::kPhiSilu;
  return q;
}

// `extra`: weight images that the call's pack launch writes as well (matrix-core path only).
int32_t history_impl(const char* fn, int phi, const void* E, const int32_t* lens, const void* LC,
                     int64_t lc_user_stride, const void* Wq, const void* Wk, const void* Wv, void* LP, void* OS,
                     int32_t B, int32_t N, int32_t d, int32_t h, int32_t m, float scale, int32_t dtype,
                     void* workspace, size_t ws_bytes, void* stream, const lime::PackWeight* extra = nullptr,
                     int n_extra = 0) {
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (N <= 0 || m <= 0) return fail(LIME_INVALID_ARG, "%s: N and m must be positive (N=%d m=%d)", fn, N, m);
  if (!E || !LC || !Wq || !Wk || !Wv || !LP) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (lc_user_stride != 0 && lc_user_stride != static_cast<int64_t>(m) * d)
    return fail(LIME_INVALID_ARG, "%s: lc_user_stride must be 0 or m*d (got %lld)", fn, static_cast<long long>(lc_user_stride));
  const bool per_user = lc_user_stride != 0;
  const bool want_os = OS != nullptr;
  // The matrix-core path: L^P / O[T] ("the m links attend over the history") on the fused history-side
  // kernel, O[S] ("every history row attends over the m links") on the candidate-side kernel with SiLU/m.
  const bool lp_on_mfma = dtype == LIME_BF16 && lime::links_over_history_supported(d, h, m) &&
                          all_aligned16(E, LC, Wq, Wk, Wv, LP, OS, workspace) && fits_tiles(B, N);
  const bool os_on_mfma = want_os && lp_on_mfma;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t link_rows = (per_user ? B : 1) * static_cast<int64_t>(m);
  const int64_t hist_rows = static_cast<int64_t>(B) * N;
  const int64_t link_stride = per_user ? static_cast<int64_t>(m) * d : 0;
  HistoryPlan p{};
  if (lp_on_mfma) {
    p.bytes = lime::links_over_history_workspace(B, N, d, h, m, per_user);
    // (when L^P runs on the matrix cores, so does O[S]: same shape and alignment conditions)
    const size_t os_bytes = os_on_mfma ? lime::queries_over_links_workspace(B, d, m, per_user) : 0;
    if (!workspace || ws_bytes < p.bytes + os_bytes)
      return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, p.bytes + os_bytes,
                  workspace ? ws_bytes : 0);
    lime::LinksOverHistory q{};
    q.E = E, q.lens = lens, q.LC = LC, q.lc_user_stride = link_stride, q.Wq = Wq, q.Wk = Wk, q.Wv = Wv, q.LP = LP;
    q.B = B, q.N = N, q.d = d, q.h = h, q.m = m, q.scale = scale, q.phi = phi;
    // one pack launch for everything this call needs on the matrix cores: the operands of both kernels and `extra`
    lime::PackJobs jobs;
    lime::links_over_history_jobs(q, workspace, jobs);
    if (os_on_mfma) lime::queries_over_links_jobs(os_query(E, lens, LC, link_stride, Wq, Wk, Wv, OS, B, N, d, h, m, scale),
                                                   static_cast<char*>(workspace) + p.bytes, jobs);
    for (int i = 0; i < n_extra; ++i) jobs.weights[jobs.n_weights++] = extra[i];
    LIME_HIP(lime::pack_operands(jobs, d, h, m, s));
    q.packed = true;
    LIME_HIP(lime::links_over_history(q, workspace, s));
  } else {
    p = plan_history(nullptr, B, N, d, m, per_user, want_os && !os_on_mfma);
    const size_t os_bytes = os_on_mfma ? lime::queries_over_links_workspace(B, d, m, per_user) : 0;
    if (!workspace || ws_bytes < p.bytes + os_bytes)
      return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, p.bytes + os_bytes,
                  workspace ? ws_bytes : 0);
    p = plan_history(workspace, B, N, d, m, per_user, want_os && !os_on_mfma);
    LIME_HIP(lime::generic_project(LC, Wq, p.Qt, link_rows, d, dtype, s));
    LIME_HIP(lime::generic_project(E, Wk, p.Ks, hist_rows, d, dtype, s));
    LIME_HIP(lime::generic_project(E, Wv, p.Vs, hist_rows, d, dtype, s));
    lime::GenericAttention t{};
    t.Q = p.Qt, t.K = p.Ks, t.V = p.Vs;
    t.q_user_stride = link_stride, t.k_user_stride = t.v_user_stride = static_cast<int64_t>(N) * d;
    t.O = LP, t.q_lens = nullptr, t.k_lens = lens;
    t.B = B, t.q_rows = m, t.n_keys = N, t.d = d, t.h = h, t.scale = scale, t.phi = phi, t.dtype = dtype;
    LIME_HIP(lime::generic_attention(t, s));
  }
  if (os_on_mfma) {
    lime::QueriesOverLinks q = os_query(E, lens, LC, link_stride, Wq, Wk, Wv, OS, B, N, d, h, m, scale);
    q.packed = true;
    LIME_HIP(lime::queries_over_links(q, static_cast<char*>(workspace) + p.bytes, s));
  } else if (want_os) {
    LIME_HIP(lime::generic_project(E, Wq, p.Qs, hist_rows, d, dtype, s));
    LIME_HIP(lime::generic_project(LC, Wk, p.Kt, link_rows, d, dtype, s));
    LIME_HIP(lime::generic_project(LC, Wv, p.Vt, link_rows, d, dtype, s));
    lime::GenericAttention o{};
    o.Q = p.Qs, o.K = p.Kt, o.V = p.Vt;
    o.q_user_stride = static_cast<int64_t>(N) * d, o.k_user_stride = o.v_user_stride = link_stride;
    o.O = OS, o.q_lens = lens, o.k_lens = nullptr;
    o.B = B, o.q_rows = N, o.n_keys = m, o.d = d, o.h = h, o.scale = scale, o.phi = lime::kPhiSilu, o.dtype = dtype;
    LIME_HIP(lime::generic_attention(o, s));
  }
  return LIME_OK;
}

// ----------------------------------------------------------------------------- candidate side (Eq. 4) and baseline (Eq. 1)
struct QueryPlan {
  float *Qt, *Kt, *Vt;
  size_t bytes;
};

QueryPlan plan_queries(void* ws, int64_t q_rows_total, int64_t k_rows_total, int64_t v_rows_total, int64_t d) {
  Arena a(ws);
  QueryPlan p{};
  p.Qt = a.take<float>(q_rows_total * d);
  p.Kt = a.take<float>(k_rows_total * d);
  p.Vt = a.take<float>(v_rows_total * d);
  p.bytes = a.used;
  return p;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int32_t lime_link_history(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride, const void* Wq,
                          const void* Wk, const void* Wv, void* LP, int32_t B, int32_t N, int32_t d, int32_t h,
                          int32_t m, float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  return history_impl("lime_link_history", lime::kPhiSoftmax, E, lens, LC, lc_user_stride, Wq, Wk, Wv, LP, nullptr, B,
                      N, d, h, m, scale, dtype, workspace, ws_bytes, stream);
}

int32_t lime_xor_history(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride, const void* Wq,
                         const void* Wk, const void* Wv, void* LP, void* OS, int32_t B, int32_t N, int32_t d,
                         int32_t h, int32_t m, float scale, int32_t dtype, void* workspace, size_t ws_bytes,
                         void* stream) {
  return history_impl("lime_xor_history", lime::kPhiSilu, E, lens, LC, lc_user_stride, Wq, Wk, Wv, LP, OS, B, N, d, h,
                      m, scale, dtype, workspace, ws_bytes, stream);
}

int32_t lime_score_candidates(const void* T, const void* L, const void* LP, const void* Wq, const void* Wk,
                              const void* Wv, void* O, int32_t B, int32_t C, int32_t d, int32_t h, int32_t m,
                              float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_score_candidates";
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (C <= 0 || m <= 0) return fail(LIME_INVALID_ARG, "%s: C and m must be positive (C=%d m=%d)", fn, C, m);
  if (!T || !L || !LP || !O) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  const int64_t q_rows = static_cast<int64_t>(B) * C, v_rows = static_cast<int64_t>(B) * m;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == LIME_BF16 && lime::queries_over_links_supported(d, h, m) &&
      all_aligned16(T, L, LP, Wq, Wk, Wv, O, workspace) && fits_tiles(B, C)) {
    const size_t need = lime::queries_over_links_workspace(B, d, m, false);
    if (!workspace || ws_bytes < need)
      return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
    lime::QueriesOverLinks q{};
    q.X = T, q.O = O, q.Wq = Wq, q.Ksrc = L, q.Wk = Wk, q.Vsrc = LP, q.Wv = Wv;
    q.k_user_stride = 0, q.v_user_stride = static_cast<int64_t>(m) * d, q.row_lens = nullptr;
    q.B = B, q.rows = C, q.d = d, q.h = h, q.m = m, q.scale = scale, q.phi = lime::kPhiSoftmax;
    LIME_HIP(lime::queries_over_links(q, workspace, s));
    return LIME_OK;
  }
  QueryPlan p = plan_queries(nullptr, q_rows, m, v_rows, d);
  if (!workspace || ws_bytes < p.bytes)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, p.bytes, workspace ? ws_bytes : 0);
  p = plan_queries(workspace, q_rows, m, v_rows, d);
  LIME_HIP(lime::generic_project(T, Wq, p.Qt, q_rows, d, dtype, s));
  LIME_HIP(lime::generic_project(L, Wk, p.Kt, m, d, dtype, s));
  LIME_HIP(lime::generic_project(LP, Wv, p.Vt, v_rows, d, dtype, s));
  lime::GenericAttention a{};
  a.Q = p.Qt, a.K = p.Kt, a.V = p.Vt;
  a.q_user_stride = static_cast<int64_t>(C) * d, a.k_user_stride = 0, a.v_user_stride = static_cast<int64_t>(m) * d;
  a.O = O, a.q_lens = nullptr, a.k_lens = nullptr;
  a.B = B, a.q_rows = C, a.n_keys = m, a.d = d, a.h = h, a.scale = scale, a.phi = lime::kPhiSoftmax, a.dtype = dtype;
  LIME_HIP(lime::generic_attention(a, s));
  return LIME_OK;
}

int32_t mha_target_attention(const void* T, const void* E, const int32_t* lens, const void* Wq, const void* Wk,
                             const void* Wv, void* O, int32_t B, int32_t C, int32_t N, int32_t d, int32_t h,
                             float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "mha_target_attention";
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (C <= 0 || N <= 0) return fail(LIME_INVALID_ARG, "%s: C and N must be positive (C=%d N=%d)", fn, C, N);
  if (!T || !E || !Wq || !Wk || !Wv || !O) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  const int64_t q_rows = static_cast<int64_t>(B) * C, k_rows = static_cast<int64_t>(B) * N;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == LIME_BF16 && lime::target_attention_supported(d, h) && all_aligned16(T, E, Wq, Wk, Wv, O, workspace) &&
      fits_tiles(B, C) && fits_tiles(B, N)) {
    const size_t need = lime::target_attention_workspace(B, C, N, d);
    if (!workspace || ws_bytes < need)
      return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
    lime::TargetAttention q{T, E, lens, Wq, Wk, Wv, O, B, C, N, d, h, scale};
    LIME_HIP(lime::target_attention(q, workspace, s));
    return LIME_OK;
  }
  QueryPlan p = plan_queries(nullptr, q_rows, k_rows, k_rows, d);
  if (!workspace || ws_bytes < p.bytes)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, p.bytes, workspace ? ws_bytes : 0);
  p = plan_queries(workspace, q_rows, k_rows, k_rows, d);
  LIME_HIP(lime::generic_project(T, Wq, p.Qt, q_rows, d, dtype, s));
  LIME_HIP(lime::generic_project(E, Wk, p.Kt, k_rows, d, dtype, s));
  LIME_HIP(lime::generic_project(E, Wv, p.Vt, k_rows, d, dtype, s));
  lime::GenericAttention a{};
  a.Q = p.Qt, a.K = p.Kt, a.V = p.Vt;
  a.q_user_stride = static_cast<int64_t>(C) * d, a.k_user_stride = a.v_user_stride = static_cast<int64_t>(N) * d;
  a.O = O, a.q_lens = nullptr, a.k_lens = lens;
  a.B = B, a.q_rows = C, a.n_keys = N, a.d = d, a.h = h, a.scale = scale, a.phi = lime::kPhiSoftmax, a.dtype = dtype;
  LIME_HIP(lime::generic_attention(a, s));
  return LIME_OK;
}

int32_t lime_build_qk_cache(const void* T, const void* L, const void* Wq, const void* Wk, void* W, int32_t B, int32_t C,
                            int32_t d, int32_t h, int32_t m, float scale, int32_t dtype, void* workspace,
                            size_t ws_bytes, void* stream) {
  const char* fn = "lime_build_qk_cache";
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (C <= 0 || m <= 0) return fail(LIME_INVALID_ARG, "%s: C and m must be positive (C=%d m=%d)", fn, C, m);
  if (!T || !L || !W) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t q_rows = static_cast<int64_t>(B) * C;
  if (dtype == LIME_BF16 && lime::queries_over_links_supported(d, h, m) && all_aligned16(T, L, Wq, Wk, W, workspace) &&
      fits_tiles(B, C) && (m * 2) % 16 == 0) {
    const size_t need = lime::queries_over_links_workspace(B, d, m, false);
    if (!workspace || ws_bytes < need)
      return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
    lime::QueriesOverLinks q{};
    q.X = T, q.O = nullptr, q.Wq = Wq, q.Ksrc = L, q.Wk = Wk, q.Vsrc = nullptr, q.Wv = nullptr;
    q.k_user_stride = 0, q.v_user_stride = 0, q.row_lens = nullptr;
    q.B = B, q.rows = C, q.d = d, q.h = h, q.m = m, q.scale = scale, q.phi = lime::kPhiSoftmax, q.weights_out = W;
    LIME_HIP(lime::queries_over_links(q, workspace, s));
    return LIME_OK;
  }
  QueryPlan p = plan_queries(nullptr, q_rows, m, 0, d);
  if (!workspace || ws_bytes < p.bytes)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, p.bytes, workspace ? ws_bytes : 0);
  p = plan_queries(workspace, q_rows, m, 0, d);
  LIME_HIP(lime::generic_project(T, Wq, p.Qt, q_rows, d, dtype, s));
  LIME_HIP(lime::generic_project(L, Wk, p.Kt, m, d, dtype, s));
  LIME_HIP(lime::generic_qk_weights(p.Qt, p.Kt, W, q_rows, d, h, m, scale, dtype, s));
  return LIME_OK;
}

namespace {

// Shared by the two online entry points of the QK-cache path: weights either per (user, candidate) or gathered
// from a table by id.
int32_t cached_impl(const char* fn, const void* W, const int32_t* ids, int32_t n_items, const void* LP, const void* Wv,
                    void* O, int32_t B, int32_t C, int32_t d, int32_t h, int32_t m, int32_t dtype, void* workspace,
                    size_t ws_bytes, void* stream) {
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (C <= 0 || m <= 0) return fail(LIME_INVALID_ARG, "%s: C and m must be positive (C=%d m=%d)", fn, C, m);
  if (!W || !LP || !O) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == LIME_BF16 && lime::queries_over_links_supported(d, h, m) && all_aligned16(W, LP, Wv, O, workspace) &&
      fits_tiles(B, C)) {
    const size_t need = lime::cached_candidates_workspace(B, d, m);
    if (!workspace || ws_bytes < need)
      return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
    lime::CachedCandidates q{W, ids, n_items, LP, Wv, O, B, C, d, h, m};
    LIME_HIP(lime::cached_candidates(q, workspace, s));
    return LIME_OK;
  }
  const int64_t v_rows = static_cast<int64_t>(B) * m;
  QueryPlan p = plan_queries(nullptr, 0, 0, v_rows, d);
  if (!workspace || ws_bytes < p.bytes)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, p.bytes, workspace ? ws_bytes : 0);
  p = plan_queries(workspace, 0, 0, v_rows, d);
  LIME_HIP(lime::generic_project(LP, Wv, p.Vt, v_rows, d, dtype, s));
  LIME_HIP(lime::generic_cached_sum(W, ids, n_items, p.Vt, O, B, C, d, h, m, dtype, s));
  return LIME_OK;
}

}  // namespace

int32_t lime_score_candidates_cached(const void* W, const void* LP, const void* Wv, void* O, int32_t B, int32_t C,
                                     int32_t d, int32_t h, int32_t m, int32_t dtype, void* workspace, size_t ws_bytes,
                                     void* stream) {
  return cached_impl("lime_score_candidates_cached", W, nullptr, 0, LP, Wv, O, B, C, d, h, m, dtype, workspace, ws_bytes,
                     stream);
}

int32_t lime_score_candidates_gathered(const void* Wtable, const int32_t* ids, int32_t n_items, const void* LP,
                                       const void* Wv, void* O, int32_t B, int32_t C, int32_t d, int32_t h, int32_t m,
                                       int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_score_candidates_gathered";
  if (!ids) return fail(LIME_INVALID_ARG, "%s: ids is NULL", fn);
  if (n_items <= 0) return fail(LIME_INVALID_ARG, "%s: n_items must be positive (%d)", fn, n_items);
  return cached_impl(fn, Wtable, ids, n_items, LP, Wv, O, B, C, d, h, m, dtype, workspace, ws_bytes, stream);
}

// ----------------------------------------------------------------------------- operands prepared once per model
size_t lime_prepared_bytes(int32_t d, int32_t h, int32_t m, int32_t dtype) {
  if (d <= 0 || h <= 0 || m <= 0 || d % h != 0 || dtype != LIME_BF16) return 0;
  if (!lime::queries_over_links_supported(d, h, m)) return 0;
  return lime::prepared_layout(d, m).total;
}

int32_t lime_prepare(const void* LC, const void* L, const void* Wq_hist, const void* Wk_hist, const void* Wv_hist,
                     const void* Wq_cand, const void* Wk_cand, float scale_hist, float scale_cand, void* prepared,
                     size_t prepared_bytes, int32_t d, int32_t h, int32_t m, int32_t dtype, void* stream) {
  const char* fn = "lime_prepare";
  if (int32_t st = check_common(fn, 1, d, h, dtype)) return st;
  if (m <= 0) return fail(LIME_INVALID_ARG, "%s: m must be positive (m=%d)", fn, m);
  if (!LC || !L || !Wq_hist || !Wk_hist || !Wv_hist || !prepared)
    return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  const size_t need = lime_prepared_bytes(d, h, m, dtype);
  if (need == 0 || !all_aligned16(LC, L, Wq_hist, Wk_hist, Wv_hist, Wq_cand, Wk_cand, prepared))
    return fail(LIME_UNSUPPORTED, "%s: prepared operands exist for the bf16 matrix-core shapes and 16-byte aligned pointers only", fn);
  if (prepared_bytes < need)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: prepared buffer of %zu bytes needed, %zu given", fn, need, prepared_bytes);
  lime::PrepareOperands p{LC, L, Wq_hist, Wk_hist, Wv_hist, Wq_cand, Wk_cand, scale_hist, scale_cand, d, h, m};
  LIME_HIP(lime::prepare_operands(p, prepared, static_cast<hipStream_t>(stream)));
  return LIME_OK;
}

int32_t lime_link_history_prepared(const void* E, const int32_t* lens, const void* prepared, void* LP, int32_t B,
                                   int32_t N, int32_t d, int32_t h, int32_t m, float scale, int32_t xor_attention,
                                   int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_link_history_prepared";
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (N <= 0 || m <= 0) return fail(LIME_INVALID_ARG, "%s: N and m must be positive (N=%d m=%d)", fn, N, m);
  if (!E || !prepared || !LP) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (lime_prepared_bytes(d, h, m, dtype) == 0 || !all_aligned16(E, prepared, LP, workspace) || !fits_tiles(B, N))
    return fail(LIME_UNSUPPORTED, "%s: prepared operands exist for the bf16 matrix-core shapes and 16-byte aligned pointers only", fn);
  const size_t need = lime::links_over_history_workspace(B, N, d, h, m, false);
  if (!workspace || ws_bytes < need)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
  lime::LinksOverHistory q{};
  q.E = E, q.lens = lens, q.LP = LP, q.prepared = prepared;
  q.B = B, q.N = N, q.d = d, q.h = h, q.m = m, q.scale = scale;
  q.phi = xor_attention ? lime::kPhiSilu : lime::kPhiSoftmax;
  LIME_HIP(lime::links_over_history(q, workspace, static_cast<hipStream_t>(stream)));
  return LIME_OK;
}

int32_t lime_score_candidates_prepared(const void* T, const void* LP, const void* Wv, const void* prepared, void* O,
                                       int32_t B, int32_t C, int32_t d, int32_t h, int32_t m, float scale,
                                       int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_score_candidates_prepared";
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (C <= 0 || m <= 0) return fail(LIME_INVALID_ARG, "%s: C and m must be positive (C=%d m=%d)", fn, C, m);
  if (!T || !LP || !prepared || !O) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (lime_prepared_bytes(d, h, m, dtype) == 0 || !all_aligned16(T, LP, Wv, prepared, O, workspace) || !fits_tiles(B, C))
    return fail(LIME_UNSUPPORTED, "%s: prepared operands exist for the bf16 matrix-core shapes and 16-byte aligned pointers only", fn);
  const size_t need = lime::queries_over_links_workspace(B, d, m, false);
  if (!workspace || ws_bytes < need)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
  lime::QueriesOverLinks q{};
  q.X = T, q.O = O, q.Vsrc = LP, q.Wv = Wv, q.prepared = prepared;
  q.k_user_stride = 0, q.v_user_stride = static_cast<int64_t>(m) * d, q.row_lens = nullptr;
  q.B = B, q.rows = C, q.d = d, q.h = h, q.m = m, q.scale = scale, q.phi = lime::kPhiSoftmax;
  LIME_HIP(lime::queries_over_links(q, workspace, static_cast<hipStream_t>(stream)));
  return LIME_OK;
}

int32_t lime_request_prepared(const void* E, const int32_t* lens, const void* T, const void* Wv, const void* prepared,
                              void* LP, void* O, int32_t B, int32_t N, int32_t C, int32_t d, int32_t h, int32_t m,
                              float scale_hist, float scale_cand, int32_t xor_attention, int32_t dtype, void* workspace,
                              size_t ws_bytes, void* stream) {
  const char* fn = "lime_request_prepared";
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (N <= 0 || C <= 0 || m <= 0)
    return fail(LIME_INVALID_ARG, "%s: N, C and m must be positive (N=%d C=%d m=%d)", fn, N, C, m);
  if (!E || !T || !prepared || !LP || !O) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (lime_prepared_bytes(d, h, m, dtype) == 0 || !all_aligned16(E, T, Wv, prepared, LP, O, workspace) || !fits_tiles(B, N) ||
      !fits_tiles(B, C))
    return fail(LIME_UNSUPPORTED, "%s: prepared operands exist for the bf16 matrix-core shapes and 16-byte aligned pointers only", fn);
  const size_t hist_bytes = lime::links_over_history_workspace(B, N, d, h, m, false);
  const size_t need = hist_bytes + lime::queries_over_links_workspace(B, d, m, false);
  if (!workspace || ws_bytes < need)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
  hipStream_t s = static_cast<hipStream_t>(stream);
  void* cand_ws = static_cast<char*>(workspace) + hist_bytes;
  lime::QueriesOverLinks c{};
  c.X = T, c.O = O, c.Vsrc = LP, c.Wv = Wv, c.prepared = prepared;
  c.k_user_stride = 0, c.v_user_stride = static_cast<int64_t>(m) * d, c.row_lens = nullptr;
  c.B = B, c.rows = C, c.d = d, c.h = h, c.m = m, c.scale = scale_cand, c.phi = lime::kPhiSoftmax;
  lime::LinksOverHistory q{};
  q.E = E, q.lens = lens, q.LP = LP, q.prepared = prepared;
  q.B = B, q.N = N, q.d = d, q.h = h, q.m = m, q.scale = scale_hist;
  q.phi = xor_attention ? lime::kPhiSilu : lime::kPhiSoftmax;
  // three kernels: the merge step of the history side also projects the finished link states and writes the value
  // image where the candidate-side kernel of this request expects it
  q.Wv_values = Wv, q.values_image = lime::queries_over_links_values(c, cand_ws);
  c.packed = true;
  LIME_HIP(lime::links_over_history(q, workspace, s));
  LIME_HIP(lime::queries_over_links(c, cand_ws, s));
  return LIME_OK;
}

namespace {

// A request's workspace: the history stage's part, then the candidate stage's.  `any_path`: both parts sized for
// whichever kernels a call of this shape could take (what lime_workspace_bytes reports); otherwise for the kernels
// this call does take.
struct RequestPlan {
  bool on_mfma;
  size_t hist_bytes, total;
};

RequestPlan plan_request(bool on_mfma, bool any_path, bool per_user, int32_t B, int32_t N, int32_t C, int32_t d, int32_t h,
                         int32_t m, int32_t dtype) {
  RequestPlan p{on_mfma, 0, 0};
  if (any_path) {
    p.hist_bytes = lime_workspace_bytes(LIME_OP_LINK_HISTORY, B, N, C, d, h, m, dtype, 0);
    p.total = p.hist_bytes + lime_workspace_bytes(LIME_OP_SCORE_CANDIDATES, B, N, C, d, h, m, dtype, 0);
  } else if (on_mfma) {
    p.hist_bytes = lime::links_over_history_workspace(B, N, d, h, m, per_user);
    p.total = p.hist_bytes + lime::queries_over_links_workspace(B, d, m, false);
  } else {
    // the two stages in turn: each picks its kernels by itself, so each part is sized for either choice
    p.hist_bytes = plan_history(nullptr, B, N, d, m, per_user, false).bytes;
    size_t cand = plan_queries(nullptr, static_cast<int64_t>(B) * C, m, static_cast<int64_t>(B) * m, d).bytes;
    if (dtype == LIME_BF16 && lime::links_over_history_supported(d, h, m)) {
      p.hist_bytes = std::max(p.hist_bytes, lime::links_over_history_workspace(B, N, d, h, m, per_user));
      cand = std::max(cand, lime::queries_over_links_workspace(B, d, m, false));
    }
    p.total = p.hist_bytes + cand;
  }
  return p;
}

int32_t check_request(const char* fn, const void* E, const void* LC, int64_t lc_user_stride, const void* Wq_hist,
                      const void* Wk_hist, const void* Wv_hist, const void* T, const void* L, void* LP, void* O, int32_t B,
                      int32_t N, int32_t C, int32_t d, int32_t h, int32_t m, int32_t dtype) {
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (N <= 0 || C <= 0 || m <= 0)
    return fail(LIME_INVALID_ARG, "%s: N, C and m must be positive (N=%d C=%d m=%d)", fn, N, C, m);
  if (!E || !LC || !Wq_hist || !Wk_hist || !Wv_hist || !T || !L || !LP || !O)
    return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (lc_user_stride != 0 && lc_user_stride != static_cast<int64_t>(m) * d)
    return fail(LIME_INVALID_ARG, "%s: lc_user_stride must be 0 or m*d (got %lld)", fn, static_cast<long long>(lc_user_stride));
  return LIME_OK;
}

// Layer normalisations applied on the way into the request's kernels (matrix-core path only): of the link rows that
// become the history stage's queries, and of the candidate stage's query, key and value rows.  (The history rows,
// which are keys and values at once, are normalised by a pass of their own before the request.)
struct RequestNorms {
  lime::RowNorm hist_q, cand_q, cand_k, cand_v;
};

// Arguments checked, workspace of p.total bytes at hand.
int32_t request_impl(const char* fn, const RequestPlan& p, const void* E, const int32_t* lens, const void* LC,
                     int64_t lc_user_stride, const void* Wq_hist, const void* Wk_hist, const void* Wv_hist, const void* T,
                     const void* L, const void* Wq_cand, const void* Wk_cand, const void* Wv_cand, void* LP, void* O,
                     int32_t B, int32_t N, int32_t C, int32_t d, int32_t h, int32_t m, float scale_hist, float scale_cand,
                     int32_t xor_attention, int32_t dtype, void* workspace, void* stream, const RequestNorms* norms = nullptr) {
  const int phi = xor_attention ? lime::kPhiSilu : lime::kPhiSoftmax;
  const bool per_user = lc_user_stride != 0;
  void* cand_ws = static_cast<char*>(workspace) + p.hist_bytes;
  if (!p.on_mfma) {  // the two stages as they are (general kernels, or the matrix-core ones where each applies)
    if (norms != nullptr) return fail(LIME_UNSUPPORTED, "%s: normalised operands need the matrix-core path", fn);
    if (int32_t st = history_impl(fn, phi, E, lens, LC, lc_user_stride, Wq_hist, Wk_hist, Wv_hist, LP, nullptr, B, N, d, h, m,
                                  scale_hist, dtype, workspace, p.hist_bytes, stream))
      return st;
    return lime_score_candidates(T, L, LP, Wq_cand, Wk_cand, Wv_cand, O, B, C, d, h, m, scale_cand, dtype, cand_ws,
                                 p.total - p.hist_bytes, stream);
  }
  // Four kernels: one pack launch for the operands of both stages, the history kernel, the merge step that also writes
  // the candidate stage's value image, the candidate kernel.
  hipStream_t s = static_cast<hipStream_t>(stream);
  lime::LinksOverHistory q{};
  q.E = E, q.lens = lens, q.LC = LC, q.lc_user_stride = per_user ? static_cast<int64_t>(m) * d : 0;
  q.Wq = Wq_hist, q.Wk = Wk_hist, q.Wv = Wv_hist, q.LP = LP;
  q.B = B, q.N = N, q.d = d, q.h = h, q.m = m, q.scale = scale_hist, q.phi = phi;
  lime::QueriesOverLinks c{};
  c.X = T, c.O = O, c.Wq = Wq_cand, c.Ksrc = L, c.Wk = Wk_cand, c.Vsrc = LP, c.Wv = Wv_cand;
  c.k_user_stride = 0, c.v_user_stride = static_cast<int64_t>(m) * d, c.row_lens = nullptr;
  c.B = B, c.rows = C, c.d = d, c.h = h, c.m = m, c.scale = scale_cand, c.phi = lime::kPhiSoftmax;
  if (norms != nullptr)
    q.q_norm = norms->hist_q, q.values_norm = norms->cand_v, c.x_norm = norms->cand_q, c.k_norm = norms->cand_k;
  lime::PackJobs jobs;
  lime::links_over_history_jobs(q, workspace, jobs);
  lime::queries_over_links_jobs(c, cand_ws, jobs, /*values=*/false);
  LIME_HIP(lime::pack_operands(jobs, d, h, m, s));
  q.packed = c.packed = true;
  q.Wv_values = Wv_cand, q.values_image = lime::queries_over_links_values(c, cand_ws);
  LIME_HIP(lime::links_over_history(q, workspace, s));
  LIME_HIP(lime::queries_over_links(c, cand_ws, s));
  return LIME_OK;
}

// ----------------------------------------------------------------------------- the request without a workspace argument
// Scratch of lime_request_static: every GPU the library runs on holds its own copy of this array, at its own
// address, until the process ends.  In host code the array's name is not a device address: the address comes from
// hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of `scratch` (looked up on the first call on that device).
int32_t static_scratch(const char* fn, void** out) {
  int dev = -1;
  LIME_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(LIME_UNSUPPORTED, "%s: device ordinal %d is beyond %d", fn, dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    LIME_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return fail(LIME_LAUNCH_FAILED, "%s: hipGetSymbolAddress returned no address", fn);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LIME_OK;
}

}  // namespace

int32_t lime_request(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride, const void* Wq_hist,
                     const void* Wk_hist, const void* Wv_hist, const void* T, const void* L, const void* Wq_cand,
                     const void* Wk_cand, const void* Wv_cand, void* LP, void* O, int32_t B, int32_t N, int32_t C,
                     int32_t d, int32_t h, int32_t m, float scale_hist, float scale_cand, int32_t xor_attention,
                     int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_request";
  if (int32_t st = check_request(fn, E, LC, lc_user_stride, Wq_hist, Wk_hist, Wv_hist, T, L, LP, O, B, N, C, d, h, m, dtype))
    return st;
  const bool on_mfma = dtype == LIME_BF16 && lime::links_over_history_supported(d, h, m) &&
                       all_aligned16(E, LC, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, LP, O, workspace) &&
                       fits_tiles(B, N) && fits_tiles(B, C);
  // each stage has a part of the workspace of its own, sized as for the stage's own entry point
  const RequestPlan p = plan_request(on_mfma, /*any_path=*/true, lc_user_stride != 0, B, N, C, d, h, m, dtype);
  if (!workspace || ws_bytes < p.total)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, p.total, workspace ? ws_bytes : 0);
  return request_impl(fn, p, E, lens, LC, lc_user_stride, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, LP, O,
                      B, N, C, d, h, m, scale_hist, scale_cand, xor_attention, dtype, workspace, stream);
}

int32_t lime_request_static(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride,
                            const void* Wq_hist, const void* Wk_hist, const void* Wv_hist, const void* T, const void* L,
                            const void* Wq_cand, const void* Wk_cand, const void* Wv_cand, void* LP, void* O, int32_t B,
                            int32_t N, int32_t C, int32_t d, int32_t h, int32_t m, float scale_hist, float scale_cand,
                            int32_t xor_attention, int32_t dtype, void* stream) {
  const char* fn = "lime_request_static";
  if (int32_t st = check_request(fn, E, LC, lc_user_stride, Wq_hist, Wk_hist, Wv_hist, T, L, LP, O, B, N, C, d, h, m, dtype))
    return st;
  const bool on_mfma = dtype == LIME_BF16 && lime::links_over_history_supported(d, h, m) &&
                       all_aligned16(E, LC, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, LP, O) &&
                       fits_tiles(B, N) && fits_tiles(B, C);
  // sized for the kernels this call takes, so that the matrix-core shapes need little
  const RequestPlan p = plan_request(on_mfma, /*any_path=*/false, lc_user_stride != 0, B, N, C, d, h, m, dtype);
  if (p.total > kStaticScratchBytes)
    return fail(LIME_UNSUPPORTED, "%s: this shape needs %zu bytes of scratch, the library's own buffer holds %zu; use lime_request with a workspace",
                fn, p.total, kStaticScratchBytes);
  void* ws = nullptr;
  if (int32_t st = static_scratch(fn, &ws)) return st;
  return request_impl(fn, p, E, lens, LC, lc_user_stride, Wq_hist, Wk_hist, Wv_hist, T, L, Wq_cand, Wk_cand, Wv_cand, LP, O,
                      B, N, C, d, h, m, scale_hist, scale_cand, xor_attention, dtype, ws, stream);
}

size_t lime_request_static_capacity(void) { return kStaticScratchBytes; }

int32_t lime_xor_layers(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride, const void* Wq,
                        const void* Wk, const void* Wv, const void* Wu, const void* Wo, int32_t n_layers, void* LP,
                        int32_t B, int32_t N, int32_t d, int32_t h, int32_t m, float scale, int32_t dtype,
                        void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_xor_layers";
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (N <= 0 || m <= 0 || n_layers <= 0)
    return fail(LIME_INVALID_ARG, "%s: N, m and n_layers must be positive (N=%d m=%d n_layers=%d)", fn, N, m, n_layers);
  if (!E || !LC || !Wq || !Wk || !Wv || !Wu || !Wo || !LP) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (lc_user_stride != 0 && lc_user_stride != static_cast<int64_t>(m) * d)
    return fail(LIME_INVALID_ARG, "%s: lc_user_stride must be 0 or m*d (got %lld)", fn, static_cast<long long>(lc_user_stride));
  // the same condition under which history_impl runs both XORA kernels on the matrix cores (the workspace pieces
  // handed to it below are 256-byte aligned)
  const bool on_mfma = dtype == LIME_BF16 && lime::links_over_history_supported(d, h, m) && fits_tiles(B, N) &&
                       all_aligned16(E, LC, Wq, Wk, Wv, Wu, Wo, LP, workspace);
  const size_t need = xor_layers_workspace(B, N, d, h, m, dtype);
  if (!workspace || ws_bytes < need)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
  const XorLayersPlan p = plan_xor_layers(workspace, B, N, d, h, m, dtype, on_mfma);
  const size_t es = dtype == LIME_BF16 ? 2 : 4;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t hist_stride = static_cast<int64_t>(N) * d, link_stride = static_cast<int64_t>(m) * d;
  const char *Wu_all = static_cast<const char*>(Wu), *Wo_all = static_cast<const char*>(Wo);
  const size_t weight_bytes = static_cast<size_t>(d) * d * es;
  for (int j = 0; j < n_layers; ++j) {
    const bool first = j == 0, last = j + 1 == n_layers;
    // the layer's inputs: the caller's tensors for the first layer, the residual stream afterwards
    const void* Ej = first ? E : p.Xs[j & 1];
    const void* Lj = first ? LC : p.Xt[j & 1];
    const int64_t lj_stride = first ? lc_user_stride : link_stride;
    // A = XORA(X_j) in block form (Eq. 7): O[T] for the link rows, O[S] for the history rows (not needed after the last layer)
    // (the layer's pack launch also writes the images of the gated block's two weights)
    const void *Wu_j = Wu_all + j * weight_bytes, *Wo_j = Wo_all + j * weight_bytes;
    lime::PackWeight images[2] = {{Wu_j, p.Wu_image}, {Wo_j, p.Wo_image}};
    if (int32_t st = history_impl(fn, lime::kPhiSilu, Ej, lens, Lj, lj_stride, Wq, Wk, Wv, p.OT, last ? nullptr : p.OS, B, N,
                                  d, h, m, scale, dtype, p.hist_ws, p.hist_bytes, stream, images, on_mfma ? 2 : 0))
      return st;
    if (!on_mfma) {
      lime::GenericGatedBlock links{};
      links.X = Lj, links.x_user_stride = lj_stride, links.Wu = Wu_j, links.Wo = Wo_j, links.A = p.OT;
      links.Y = last ? nullptr : p.Xt[(j + 1) & 1];
      links.sum_in = first ? nullptr : p.sum, links.sum_out = last ? nullptr : p.sum, links.sum_rounded = last ? LP : nullptr;
      links.P = p.P, links.Z = p.Z, links.B = B, links.rows = m, links.d = d, links.dtype = dtype;
      LIME_HIP(lime::generic_gated_block(links, s));
      if (last) break;
      lime::GenericGatedBlock rows{};
      rows.X = Ej, rows.x_user_stride = hist_stride, rows.lens = lens, rows.Wu = Wu_j, rows.Wo = Wo_j, rows.A = p.OS;
      rows.Y = p.Xs[(j + 1) & 1], rows.P = p.P, rows.Z = p.Z, rows.B = B, rows.rows = N, rows.d = d, rows.dtype = dtype;
      LIME_HIP(lime::generic_gated_block(rows, s));
      continue;
    }
    // link rows: Y = (O[T] * SiLU(X Wu)) Wo joins the running sum (= L^P after the last layer) and the stream
    lime::GatedBlock links{};
    links.X = Lj, links.x_user_stride = lj_stride, links.Wu_image = p.Wu_image, links.Wo_image = p.Wo_image, links.A = p.OT;
    links.B = B, links.rows = m, links.d = d, links.h = h;
    links.Y = last ? nullptr : p.Xt[(j + 1) & 1];
    links.sum_in = first ? nullptr : p.sum, links.sum_out = last ? nullptr : p.sum, links.sum_rounded = last ? LP : nullptr;
    LIME_HIP(lime::gated_block(links, s));
    if (last) break;
    // history rows: the same block with O[S]; rows at or past lens[b] stay zero
    lime::GatedBlock rows{};
    rows.X = Ej, rows.x_user_stride = hist_stride, rows.lens = lens, rows.Wu_image = p.Wu_image, rows.Wo_image = p.Wo_image;
    rows.A = p.OS, rows.Y = p.Xs[(j + 1) & 1], rows.B = B, rows.rows = N, rows.d = d, rows.h = h;
    LIME_HIP(lime::gated_block(rows, s));
  }
  return LIME_OK;
}

int32_t lime_xor_backward(const void* QS, const void* KS, const void* VS, const void* QT, const void* KT, const void* VT,
                          const void* dOT, const void* dOS, const int32_t* lens, void* dQS, void* dKS, void* dVS,
                          void* dQT, void* dKT, void* dVT, int32_t B, int32_t N, int32_t m, int32_t d, int32_t h,
                          float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_xor_backward";
  if (int32_t st = check_common(fn, B, d, h, dtype)) return st;
  if (N <= 0 || m <= 0) return fail(LIME_INVALID_ARG, "%s: N and m must be positive (N=%d m=%d)", fn, N, m);
  if (!QS || !KS || !VS || !QT || !KT || !VT || !dOT || !dQS || !dKS || !dVS || !dQT || !dKT || !dVT)
    return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (!lime::xor_backward_supported(d, h))
    return fail(LIME_UNSUPPORTED, "%s: head width d/h = %d is beyond the %d this kernel is built for", fn, d / h, 64);
  const size_t need = lime::xor_backward_workspace(B, N, m, d, h);
  if (!workspace || ws_bytes < need)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
  lime::XorBackward g{};
  g.QS = QS, g.KS = KS, g.VS = VS, g.QT = QT, g.KT = KT, g.VT = VT, g.dOT = dOT, g.dOS = dOS, g.lens = lens;
  g.dQS = dQS, g.dKS = dKS, g.dVS = dVS, g.dQT = dQT, g.dKT = dKT, g.dVT = dVT;
  g.B = B, g.N = N, g.m = m, g.d = d, g.h = h, g.dtype = dtype, g.scale = scale;
  LIME_HIP(lime::xor_backward(g, workspace, static_cast<hipStream_t>(stream)));
  return LIME_OK;
}


// ----------------------------------------------------------------------------- the scoring pipeline around the attention stages
namespace {

constexpr int kMaxMlpMaps = 4;

int32_t check_mlp(const char* fn, const void* const* W, const void* const* b, const int32_t* widths, int32_t n_maps, int32_t d) {
  if (!W || !b || !widths) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (n_maps < 1 || n_maps > kMaxMlpMaps)
    return fail(LIME_INVALID_ARG, "%s: the interaction network has 1 to %d affine maps (got %d)", fn, kMaxMlpMaps, n_maps);
  for (int i = 0; i < n_maps; ++i) {
    if (widths[i] <= 0 || !W[i]) return fail(LIME_INVALID_ARG, "%s: map %d has no weights or a non-positive width", fn, i);
  }
  if (widths[n_maps - 1] != 1) return fail(LIME_INVALID_ARG, "%s: the last map must produce one logit (width %d)", fn, widths[n_maps - 1]);
  if (d <= 0) return fail(LIME_INVALID_ARG, "%s: d must be positive", fn);
  return LIME_OK;
}

bool mlp_on_mfma(const void* O, const void* const* W, const void* const* b, const int32_t* widths, int32_t n_maps, int32_t d,
                 int32_t dtype, const void* workspace) {
  if (dtype != LIME_BF16 || !lime::interaction_mlp_on_matrix_cores(d, n_maps, widths) || !all_aligned16(O, workspace)) return false;
  for (int i = 0; i < n_maps; ++i)
    if ((reinterpret_cast<uintptr_t>(W[i]) | reinterpret_cast<uintptr_t>(b[i])) & 1u) return false;
  return true;
}

size_t mlp_workspace(int64_t rows, int32_t d, const int32_t* widths, int32_t n_maps, int32_t dtype) {
  int widest = 1;
  for (int i = 0; i < n_maps; ++i) widest = std::max(widest, widths[i]);
  // general kernels: two fp32 buffers of rows x the widest layer, used in turn
  size_t need = 2 * lime::align_up(static_cast<size_t>(rows) * widest * sizeof(float));
  if (dtype == LIME_BF16 && lime::interaction_mlp_on_matrix_cores(d, n_maps, widths))
    need = std::max(need, lime::interaction_mlp_image_bytes(d, n_maps, widths));
  return need;
}

int32_t mlp_impl(const char* fn, const void* O, const void* const* W, const void* const* b, const int32_t* widths, int32_t n_maps,
                 float* scores, int64_t rows, int32_t d, int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  const size_t need = mlp_workspace(rows, d, widths, n_maps, dtype);
  if (!workspace || ws_bytes < need)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (mlp_on_mfma(O, W, b, widths, n_maps, d, dtype, workspace)) {
    LIME_HIP(lime::interaction_mlp_mfma(O, rows, d, n_maps, widths, W, b, scores, workspace, s));
    return LIME_OK;
  }
  int widest = 1;
  for (int i = 0; i < n_maps; ++i) widest = std::max(widest, widths[i]);
  float* buf[2] = {static_cast<float*>(workspace),
                   reinterpret_cast<float*>(static_cast<char*>(workspace) + lime::align_up(static_cast<size_t>(rows) * widest * sizeof(float)))};
  const void* x = O;
  int din = d, x_dtype = dtype;
  for (int i = 0; i < n_maps; ++i) {
    const bool last = i + 1 == n_maps;
    lime::Dense q{};
    q.X1 = x, q.W = W[i], q.b = b[i], q.Y = last ? static_cast<void*>(scores) : static_cast<void*>(buf[i & 1]);
    q.rows = rows, q.d1 = din, q.dout = widths[i], q.relu = !last;
    q.x_dtype = x_dtype, q.w_dtype = dtype, q.y_dtype = LIME_F32;
    LIME_HIP(lime::dense_rows(q, s));
    x = buf[i & 1], din = widths[i], x_dtype = LIME_F32;
  }
  return LIME_OK;
}

int32_t contextualize_impl(const char* fn, const void* L, const void* EC, const void* W1, const void* b1, const void* W2,
                           const void* b2, void* LC, int32_t B, int32_t m, int32_t d, int32_t dc, int32_t dhid, int32_t dtype,
                           void* workspace, size_t ws_bytes, void* stream) {
  const size_t need = lime::align_up(static_cast<size_t>(B) * m * dhid * sizeof(float));
  if (!workspace || ws_bytes < need)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace ? ws_bytes : 0);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t rows = static_cast<int64_t>(B) * m;
  lime::Dense h{};  // hidden = ReLU([L | E^C_b] W1 + b1)
  h.X1 = L, h.x1_rows = m, h.X2 = EC, h.x2_rows_per = m, h.W = W1, h.b = b1, h.Y = workspace;
  h.rows = rows, h.d1 = d, h.d2 = dc, h.dout = dhid, h.relu = true, h.x_dtype = dtype, h.w_dtype = dtype, h.y_dtype = LIME_F32;
  LIME_HIP(lime::dense_rows(h, s));
  lime::Dense o{};  // L^C = hidden W2 + b2
  o.X1 = workspace, o.W = W2, o.b = b2, o.Y = LC;
  o.rows = rows, o.d1 = dhid, o.dout = d, o.relu = false, o.x_dtype = LIME_F32, o.w_dtype = dtype, o.y_dtype = dtype;
  LIME_HIP(lime::dense_rows(o, s));
  return LIME_OK;
}

struct ScoresPlan {
  size_t LC, hid, En, LCn, Tn, Ln, LP, LPn, O, hist, cand, mlp, total;
  size_t hist_bytes, cand_bytes, mlp_bytes, hid_bytes;
};

ScoresPlan plan_scores(const lime_scoring_model& M, int32_t B, int32_t N, int32_t C, int32_t dtype) {
  ScoresPlan p{};
  const size_t es = dtype == LIME_BF16 ? 2 : 4;
  const size_t links = lime::align_up(static_cast<size_t>(B) * M.m * M.d * es);
  size_t at = 0;
  auto take = [&](size_t bytes) { const size_t o = at; at += lime::align_up(bytes); return o; };
  p.LC = take(links);
  p.hid_bytes = lime::align_up(static_cast<size_t>(B) * M.m * M.dhid * sizeof(float));
  p.hid = take(p.hid_bytes);
  p.En = take(static_cast<size_t>(B) * N * M.d * es);
  p.LCn = take(links);
  p.Tn = take(static_cast<size_t>(B) * C * M.d * es);
  p.Ln = take(static_cast<size_t>(M.m) * M.d * es);
  p.LP = take(links);
  p.LPn = take(links);
  p.O = take(static_cast<size_t>(B) * C * M.d * es);
  // the two attention stages' scratch, laid out as a request's (the history stage's part, then the candidate stage's)
  const RequestPlan r = plan_request(false, /*any_path=*/true, true, B, N, C, M.d, M.h, M.m, dtype);
  p.hist_bytes = r.hist_bytes, p.cand_bytes = r.total - r.hist_bytes;
  p.hist = take(r.total);
  p.cand = p.hist + p.hist_bytes;
  p.mlp_bytes = mlp_workspace(static_cast<int64_t>(B) * C, M.d, M.mlp_width, M.n_mlp, dtype);
  p.mlp = take(p.mlp_bytes);
  p.total = at;
  return p;
}

int32_t check_scoring_model(const char* fn, const lime_scoring_model* M, int32_t dtype) {
  if (!M) return fail(LIME_INVALID_ARG, "%s: model is NULL", fn);
  if (int32_t st = check_common(fn, 1, M->d, M->h, dtype)) return st;
  if (M->m <= 0 || M->dc <= 0 || M->dhid <= 0)
    return fail(LIME_INVALID_ARG, "%s: m, dc and dhid must be positive (m=%d dc=%d dhid=%d)", fn, M->m, M->dc, M->dhid);
  if (!M->L || !M->ctx_W1 || !M->ctx_W2 || !M->hist_Wq || !M->hist_Wk || !M->hist_Wv || !M->cand_Wq || !M->cand_Wk || !M->cand_Wv)
    return fail(LIME_INVALID_ARG, "%s: a required pointer of the model is NULL", fn);
  if (!(M->ln_eps >= 0.f)) return fail(LIME_INVALID_ARG, "%s: ln_eps must not be negative", fn);
  return check_mlp(fn, M->mlp_W, M->mlp_b, M->mlp_width, M->n_mlp, M->d);
}

}  // namespace

int32_t lime_layer_norm(const void* X, const void* gamma, const void* beta, float eps, void* Y, int64_t rows, int32_t d,
                        int32_t dtype, void* stream) {
  const char* fn = "lime_layer_norm";
  if (dtype != LIME_F32 && dtype != LIME_BF16) return fail(LIME_INVALID_ARG, "%s: unknown dtype %d", fn, dtype);
  if (rows <= 0 || d <= 0) return fail(LIME_INVALID_ARG, "%s: rows and d must be positive (rows=%lld d=%d)", fn, static_cast<long long>(rows), d);
  if (!X || !Y) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (!(eps >= 0.f)) return fail(LIME_INVALID_ARG, "%s: eps must not be negative", fn);
  LIME_HIP(lime::layer_norm_rows(X, gamma, beta, eps, Y, rows, d, nullptr, 1, dtype, static_cast<hipStream_t>(stream)));
  return LIME_OK;
}

int32_t lime_contextualize_links(const void* L, const void* EC, const void* W1, const void* b1, const void* W2, const void* b2,
                                 void* LC, int32_t B, int32_t m, int32_t d, int32_t dc, int32_t dhid, int32_t dtype,
                                 void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_contextualize_links";
  if (dtype != LIME_F32 && dtype != LIME_BF16) return fail(LIME_INVALID_ARG, "%s: unknown dtype %d", fn, dtype);
  if (B <= 0 || m <= 0 || d <= 0 || dc <= 0 || dhid <= 0)
    return fail(LIME_INVALID_ARG, "%s: B, m, d, dc, dhid must be positive (B=%d m=%d d=%d dc=%d dhid=%d)", fn, B, m, d, dc, dhid);
  if (!L || !EC || !W1 || !W2 || !LC) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  return contextualize_impl(fn, L, EC, W1, b1, W2, b2, LC, B, m, d, dc, dhid, dtype, workspace, ws_bytes, stream);
}

size_t lime_interaction_mlp_workspace_bytes(int64_t rows, int32_t d, const int32_t* widths, int32_t n_maps, int32_t dtype) {
  if (rows <= 0 || d <= 0 || !widths || n_maps < 1 || n_maps > kMaxMlpMaps || (dtype != LIME_F32 && dtype != LIME_BF16)) return 0;
  for (int i = 0; i < n_maps; ++i)
    if (widths[i] <= 0) return 0;
  return mlp_workspace(rows, d, widths, n_maps, dtype);
}

int32_t lime_interaction_mlp(const void* O, const void* const* W, const void* const* b, const int32_t* widths, int32_t n_maps,
                             float* scores, int64_t rows, int32_t d, int32_t dtype, void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_interaction_mlp";
  if (dtype != LIME_F32 && dtype != LIME_BF16) return fail(LIME_INVALID_ARG, "%s: unknown dtype %d", fn, dtype);
  if (rows <= 0) return fail(LIME_INVALID_ARG, "%s: rows must be positive", fn);
  if (!O || !scores) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  if (int32_t st = check_mlp(fn, W, b, widths, n_maps, d)) return st;
  return mlp_impl(fn, O, W, b, widths, n_maps, scores, rows, d, dtype, workspace, ws_bytes, stream);
}

size_t lime_scores_workspace_bytes(const lime_scoring_model* model, int32_t B, int32_t N, int32_t C, int32_t dtype) {
  if (!model || B <= 0 || N <= 0 || C <= 0 || model->d <= 0 || model->h <= 0 || model->m <= 0 || model->dc <= 0 || model->dhid <= 0 ||
      model->d % model->h != 0 || model->n_mlp < 1 || model->n_mlp > kMaxMlpMaps || (dtype != LIME_F32 && dtype != LIME_BF16))
    return 0;
  for (int i = 0; i < model->n_mlp; ++i)
    if (model->mlp_width[i] <= 0) return 0;
  return plan_scores(*model, B, N, C, dtype).total;
}

int32_t lime_scores(const lime_scoring_model* model, const void* E, const int32_t* lens, const void* EC, const void* T,
                    void* LC, void* LP, void* O, float* scores, int32_t B, int32_t N, int32_t C, int32_t dtype,
                    void* workspace, size_t ws_bytes, void* stream) {
  const char* fn = "lime_scores";
  if (int32_t st = check_scoring_model(fn, model, dtype)) return st;
  if (int32_t st = check_common(fn, B, model->d, model->h, dtype)) return st;
  if (N <= 0 || C <= 0) return fail(LIME_INVALID_ARG, "%s: N and C must be positive (N=%d C=%d)", fn, N, C);
  if (!E || !EC || !T || !scores) return fail(LIME_INVALID_ARG, "%s: a required pointer is NULL", fn);
  const lime_scoring_model& M = *model;
  const ScoresPlan p = plan_scores(M, B, N, C, dtype);
  if (!workspace || ws_bytes < p.total)
    return fail(LIME_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", fn, p.total, workspace ? ws_bytes : 0);
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(LIME_INVALID_ARG, "%s: the workspace must be 256-byte aligned", fn);
  char* ws = static_cast<char*>(workspace);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int d = M.d, m = M.m;
  void* lc = LC ? LC : ws + p.LC;
  void* lp = LP ? LP : ws + p.LP;
  void* o = O ? O : ws + p.O;
  // Eq. 2
  if (int32_t st = contextualize_impl(fn, M.L, EC, M.ctx_W1, M.ctx_b1, M.ctx_W2, M.ctx_b2, lc, B, m, d, M.dc, M.dhid, dtype,
                                      ws + p.hid, p.hid_bytes, stream))
    return st;
  // Eq. 3 on normalised inputs (history rows past lens[b] are skipped: nothing reads them)
  LIME_HIP(lime::layer_norm_rows(E, M.ln_hist_kv[0], M.ln_hist_kv[1], M.ln_eps, ws + p.En, static_cast<int64_t>(B) * N, d, lens, N, dtype, s));
  const int64_t link_stride = static_cast<int64_t>(m) * d;
  const bool on_mfma = dtype == LIME_BF16 && lime::links_over_history_supported(d, M.h, m) && fits_tiles(B, N) && fits_tiles(B, C) &&
                       all_aligned16(E, T, M.L, lc, lp, o, M.hist_Wq, M.hist_Wk, M.hist_Wv, M.cand_Wq, M.cand_Wk, M.cand_Wv) &&
                       // (the kernels that normalise on the way in fetch scale and shift unconditionally, 16 bytes at a time)
                       M.ln_hist_q[0] && M.ln_hist_q[1] && M.ln_cand_q[0] && M.ln_cand_q[1] && M.ln_cand_k[0] && M.ln_cand_k[1] &&
                       M.ln_cand_v[0] && M.ln_cand_v[1] &&
                       all_aligned16(M.ln_hist_q[0], M.ln_hist_q[1], M.ln_cand_q[0], M.ln_cand_q[1], M.ln_cand_k[0], M.ln_cand_k[1],
                                     M.ln_cand_v[0], M.ln_cand_v[1]);
  if (on_mfma) {
    // The request's four kernels with the other four normalisations inside them: the link rows L^C and L as the pack
    // step reads them, the finished link states L^P as the merge step projects them, the candidate rows as the
    // candidate kernel parks their tiles.  Each rounds to bf16 where the separate pass would have stored its result.
    RequestNorms norms;
    norms.hist_q = {true, M.ln_hist_q[0], M.ln_hist_q[1], M.ln_eps};
    norms.cand_q = {true, M.ln_cand_q[0], M.ln_cand_q[1], M.ln_eps};
    norms.cand_k = {true, M.ln_cand_k[0], M.ln_cand_k[1], M.ln_eps};
    norms.cand_v = {true, M.ln_cand_v[0], M.ln_cand_v[1], M.ln_eps};
    RequestPlan r = plan_request(true, /*any_path=*/true, true, B, N, C, d, M.h, m, dtype);
    if (int32_t st = request_impl(fn, r, ws + p.En, lens, lc, link_stride, M.hist_Wq, M.hist_Wk, M.hist_Wv, T, M.L, M.cand_Wq,
                                  M.cand_Wk, M.cand_Wv, lp, o, B, N, C, d, M.h, m, M.scale_hist, M.scale_cand, 0, dtype,
                                  ws + p.hist, stream, &norms))
      return st;
  } else {
    LIME_HIP(lime::layer_norm_rows(lc, M.ln_hist_q[0], M.ln_hist_q[1], M.ln_eps, ws + p.LCn, static_cast<int64_t>(B) * m, d, nullptr, 1, dtype, s));
    if (int32_t st = history_impl(fn, lime::kPhiSoftmax, ws + p.En, lens, ws + p.LCn, link_stride, M.hist_Wq, M.hist_Wk,
                                  M.hist_Wv, lp, nullptr, B, N, d, M.h, m, M.scale_hist, dtype, ws + p.hist, p.hist_bytes, stream))
      return st;
    // Eq. 4 on normalised inputs: keys from the raw links, values from the personalised links
    LIME_HIP(lime::layer_norm_rows(T, M.ln_cand_q[0], M.ln_cand_q[1], M.ln_eps, ws + p.Tn, static_cast<int64_t>(B) * C, d, nullptr, 1, dtype, s));
    LIME_HIP(lime::layer_norm_rows(M.L, M.ln_cand_k[0], M.ln_cand_k[1], M.ln_eps, ws + p.Ln, m, d, nullptr, 1, dtype, s));
    LIME_HIP(lime::layer_norm_rows(lp, M.ln_cand_v[0], M.ln_cand_v[1], M.ln_eps, ws + p.LPn, static_cast<int64_t>(B) * m, d, nullptr, 1, dtype, s));
    if (int32_t st = lime_score_candidates(ws + p.Tn, ws + p.Ln, ws + p.LPn, M.cand_Wq, M.cand_Wk, M.cand_Wv, o, B, C, d, M.h, m,
                                           M.scale_cand, dtype, ws + p.cand, p.cand_bytes, stream))
      return st;
  }
  // Section 3.3: the interaction network
  return mlp_impl(fn, o, M.mlp_W, M.mlp_b, M.mlp_width, M.n_mlp, scores, static_cast<int64_t>(B) * C, d, dtype, ws + p.mlp, p.mlp_bytes, stream);
}

size_t lime_workspace_bytes(int32_t op, int32_t B, int32_t N, int32_t C, int32_t d, int32_t h, int32_t m,
                            int32_t dtype, int32_t flags) {
  if (B <= 0 || d <= 0 || h <= 0 || d % h != 0 || d / h > kMaxHeadDim || B > kMaxUsers) return 0;
  if (dtype != LIME_F32 && dtype != LIME_BF16) return 0;
  switch (op) {
    case LIME_OP_LINK_HISTORY:
    case LIME_OP_XOR_HISTORY:
      if (N <= 0 || m <= 0) return 0;
      // sized for per-user links, the larger of the two link layouts
    {
      const bool os = op == LIME_OP_XOR_HISTORY && (flags & 1);
      size_t need = plan_history(nullptr, B, N, d, m, true, os).bytes;
      if (dtype == LIME_BF16 && lime::links_over_history_supported(d, h, m))
        need = std::max(need, lime::links_over_history_workspace(B, N, d, h, m, true) +
                                  (os ? lime::queries_over_links_workspace(B, d, m, true) : size_t{0}));
      return need;
    }
    case LIME_OP_XOR_BACKWARD:
      if (N <= 0 || m <= 0 || !lime::xor_backward_supported(d, h)) return 0;
      return lime::xor_backward_workspace(B, N, m, d, h);
    case LIME_OP_REQUEST:
      if (N <= 0 || C <= 0 || m <= 0) return 0;
      return lime_workspace_bytes(LIME_OP_LINK_HISTORY, B, N, C, d, h, m, dtype, 0) +
             lime_workspace_bytes(LIME_OP_SCORE_CANDIDATES, B, N, C, d, h, m, dtype, 0);
    case LIME_OP_REQUEST_PREPARED:
      if (N <= 0 || C <= 0 || m <= 0 || lime_prepared_bytes(d, h, m, dtype) == 0) return 0;
      return lime::links_over_history_workspace(B, N, d, h, m, false) + lime::queries_over_links_workspace(B, d, m, false);
    case LIME_OP_XOR_LAYERS:
      if (N <= 0 || m <= 0) return 0;
      return xor_layers_workspace(B, N, d, h, m, dtype);
    case LIME_OP_SCORE_CANDIDATES:
      if (C <= 0 || m <= 0) return 0;
      return std::max(plan_queries(nullptr, static_cast<int64_t>(B) * C, m, static_cast<int64_t>(B) * m, d).bytes,
                      dtype == LIME_BF16 && lime::queries_over_links_supported(d, h, m)
                          ? lime::queries_over_links_workspace(B, d, m, false) : size_t{0});
    case LIME_OP_MHA_TARGET:
      if (C <= 0 || N <= 0) return 0;
      return std::max(plan_queries(nullptr, static_cast<int64_t>(B) * C, static_cast<int64_t>(B) * N, static_cast<int64_t>(B) * N, d).bytes,
                      dtype == LIME_BF16 && lime::target_attention_supported(d, h)
                          ? lime::target_attention_workspace(B, C, N, d) : size_t{0});
    case LIME_OP_BUILD_QK_CACHE:
      if (C <= 0 || m <= 0) return 0;
      return std::max(plan_queries(nullptr, static_cast<int64_t>(B) * C, m, 0, d).bytes,
                      dtype == LIME_BF16 && lime::queries_over_links_supported(d, h, m)
                          ? lime::queries_over_links_workspace(B, d, m, false) : size_t{0});
    case LIME_OP_SCORE_CACHED:
      if (C <= 0 || m <= 0) return 0;
      return std::max(plan_queries(nullptr, 0, 0, static_cast<int64_t>(B) * m, d).bytes,
                      dtype == LIME_BF16 && lime::queries_over_links_supported(d, h, m)
                          ? lime::cached_candidates_workspace(B, d, m) : size_t{0});
    default:
      return 0;
  }
}

const char* lime_last_error(void) { return g_error; }

const char* lime_version(void) { return "0.1.0"; }

#pragma GCC visibility pop
}  // extern "C"
