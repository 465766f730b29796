/*
 * lime.h - C ABI of the MI355X (gfx950) LIME inference hot path, arXiv 2510.18239.
 *
 * Conventions common to every entry point
 * ---------------------------------------
 * Pointers.  Every tensor pointer is a DEVICE pointer owned by the caller.  The
 *   entry points never allocate, free, copy to the host or synchronise (the one
 *   exception is the benchmark's timing helper at the end of this file:
 *   lime_profile_enable makes launches create HIP events, lime_profile_collect
 *   waits for them; lime_request_many keeps a few host threads, no GPU resource).
 *   `lens` is a device pointer too.  Outputs must not alias inputs.
 * Layout.  Row-major, innermost dimension contiguous, no padding between rows:
 *   E[B][N][d], T[B][C][d], L[m][d], LP[B][m][d], W[d_in][d_out] (so that the
 *   projection of Eq. 1 is X~ = X W).
 * dtype.  LIME_F32 (0) or LIME_BF16 (1); it applies to every tensor argument
 *   and every output of the call.  Products are accumulated in fp32; bf16
 *   outputs are rounded to nearest-even from the fp32 accumulators.
 * Heads.  The d projected columns are cut into h contiguous blocks of d/h; heads
 *   are independent and their outputs concatenated; there is no output
 *   projection (theta = {W_Q, W_K, W_V} only, Eq. 1).
 * scale.  Multiplies every logit before phi ("scaled softmax", Eq. 1).  Callers
 *   normally pass (d/h)^-1/2 for the softmax paths and 1 for XORA (Algorithm 2
 *   applies SiLU to the raw product).
 * Ragged histories.  lens[b] in [0, N] is the number of valid history rows of
 *   user b (NULL = all N).  Rows at or beyond lens[b] are never read into any
 *   result: they may hold anything, NaN included.  The result for user b equals
 *   the result on E[b] truncated to lens[b] rows; a user with lens[b] = 0 gets
 *   all-zero outputs.  lens[b] outside [0, N] is a contract violation that is
 *   not checked on the device.
 * workspace.  Scratch device memory of at least lime_workspace_bytes(...) bytes,
 *   256-byte aligned, private to the call until the stream has passed it.
 * stream.  A hipStream_t passed as void* (NULL = the default stream).  All work
 *   is enqueued on it, in order.
 * Status.  0 LIME_OK; 1 LIME_INVALID_ARG (a required pointer is NULL, a
 *   dimension is <= 0, d % h != 0, unknown dtype); 2 LIME_UNSUPPORTED (shape
 *   outside the limits below); 3 LIME_WORKSPACE_TOO_SMALL; 4 LIME_LAUNCH_FAILED
 *   (a HIP error; text in lime_last_error()).  Arguments are checked on the host
 *   before anything is launched, so on any non-zero status nothing was enqueued
 *   (except LIME_LAUNCH_FAILED, where earlier launches of the call may have been).
 * Limits.  d/h <= 256.  The bf16 matrix-core (MFMA) kernels serve d/h in {32, 64}
 *   with h in {1, 2, 4, 8}, d <= 256 and m a multiple of 32 up to 128; every other
 *   shape, and all of fp32, runs on the general fp32-arithmetic kernels.
 *   lime_xor_backward: d/h <= 64; its matrix-core form serves bf16 with d/h in {32, 64}, any h and m.
 */
#ifndef LIME_H_
#define LIME_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { LIME_OK = 0, LIME_INVALID_ARG = 1, LIME_UNSUPPORTED = 2, LIME_WORKSPACE_TOO_SMALL = 3, LIME_LAUNCH_FAILED = 4 };
enum { LIME_F32 = 0, LIME_BF16 = 1 };
enum { LIME_OP_LINK_HISTORY = 0, LIME_OP_XOR_HISTORY = 1, LIME_OP_SCORE_CANDIDATES = 2, LIME_OP_MHA_TARGET = 3,
       LIME_OP_BUILD_QK_CACHE = 4, LIME_OP_SCORE_CACHED = 5, LIME_OP_XOR_LAYERS = 6, LIME_OP_REQUEST_PREPARED = 7,
       LIME_OP_REQUEST = 8, LIME_OP_XOR_BACKWARD = 9 };

/*
 * User-side link personalisation, Section 3.1 Eq. 3:
 *   LP[b] = MHA(LC_b, E[b], E[b]; J; theta),  phi = softmax over the valid history rows.
 * LC: contextualised links L^C (the output of Eq. 2, taken as given).  User b's links
 *   start at LC + b * lc_user_stride elements: 0 = one [m][d] set shared by all users,
 *   m*d = a [B][m][d] tensor.
 * Out: LP[B][m][d].
 */
int32_t lime_link_history(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride,
                          const void* Wq, const void* Wk, const void* Wv, void* LP,
                          int32_t B, int32_t N, int32_t d, int32_t h, int32_t m,
                          float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream);

/*
 * One XOR-attention layer, Section 3.2 Eq. 6-7, Appendix H.1, Appendix I Algorithms 1-2.
 * Source = the user's lens[b] valid history rows, target = the m links, one theta for both:
 *   LP[b] = O[T] = (1/n_s) SiLU(scale * Q[T] K[S]^T) V[S],   n_s = lens[b]
 *   OS[b] = O[S] = (1/n_t) SiLU(scale * Q[S] K[T]^T) V[T],   n_t = m
 * with Q[S], K[S], V[S] = E[b] Wq, Wk, Wv and Q[T], K[T], V[T] = LC_b Wq, Wk, Wv, per head.
 * Out: LP[B][m][d]; OS[B][N][d] when OS != NULL (rows >= lens[b] are written as zeros).
 */
int32_t lime_xor_history(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride,
                         const void* Wq, const void* Wk, const void* Wv, void* LP, void* OS,
                         int32_t B, int32_t N, int32_t d, int32_t h, int32_t m,
                         float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream);

/*
 * LIME-XOR's user side with n stacked XOR layers, Section 3.2 Eq. 8:
 *   LP[b] = sum_j GatedMLP(XORA(X_j, X_j, X_j; theta); eta_j) on the link rows,   X_1 = E[b] (+) LC_b.
 * XORA is the layer lime_xor_history computes (Eq. 6-7, one theta = Wq, Wk, Wv for all layers).  The paper names
 * GatedMLP ("an MLP block that learns a gated element-wise product") and the stacking without defining them; this
 * library takes GatedMLP(A; eta)(X) = (A * SiLU(X Wu)) Wo with eta_j = (Wu[j], Wo[j]), each [d][d], applied row by
 * row to history and link rows alike, and a residual stream X_{j+1} = X_j + GatedMLP(...) between the layers.
 * In: E, lens, LC, lc_user_stride, Wq, Wk, Wv as for lime_xor_history; Wu[n_layers][d][d], Wo[n_layers][d][d].
 * Out: LP[B][m][d] (zeros for a user without history).  Intermediate tensors live in the workspace
 * (LIME_OP_XOR_LAYERS) in the storage type; the link outputs are summed in fp32.
 */
int32_t lime_xor_layers(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride,
                        const void* Wq, const void* Wk, const void* Wv, const void* Wu, const void* Wo, int32_t n_layers,
                        void* LP, int32_t B, int32_t N, int32_t d, int32_t h, int32_t m,
                        float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream);

/*
 * Candidate-side decoupled attention, Section 3.1 Eq. 4 and Section 3.3:
 *   O[b] = MHA(T[b], L, LP[b]; J; theta),  phi = softmax over the m links;
 * the keys are the raw, user-independent links L[m][d], the values the personalised
 * links LP[B][m][d].  Each of Wq, Wk, Wv may be NULL (= identity), which yields the
 * literal right-hand side phi(T L^t) L^P.
 * Out: O[B][C][d].
 */
int32_t lime_score_candidates(const void* T, const void* L, const void* LP,
                              const void* Wq, const void* Wk, const void* Wv, void* O,
                              int32_t B, int32_t C, int32_t d, int32_t h, int32_t m,
                              float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream);

/*
 * Baseline: full target attention (the "MHA skyline", Section 4.1), Eq. 1 with the
 * candidates as queries and the history as keys and values:
 *   O[b] = MHA(T[b], E[b], E[b]; M; theta),  M = valid history rows, phi = softmax.
 * Out: O[B][C][d].
 */
int32_t mha_target_attention(const void* T, const void* E, const int32_t* lens,
                             const void* Wq, const void* Wk, const void* Wv, void* O,
                             int32_t B, int32_t C, int32_t N, int32_t d, int32_t h,
                             float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream);

/*
 * The three-stage inference of Section 3.3 ("QK cache").  The attention weights of Eq. 4 depend on the
 * candidate and on the raw links only, not on the user, so they can be computed ahead of time:
 *   lime_build_qk_cache:  W[b][c][a][i] = softmax over the m links i of scale * <(T[b][c] Wq)_a, (L Wk)[i]_a>
 *     (offline item side).  Out: W[B][C][h][m] in `dtype`.  Wq, Wk may be NULL (identity).
 *   lime_score_candidates_cached:  O[b][c][head a] = sum_i W[b][c][a][i] * (LP[b] Wv)[i][head a]
 *     (online: a lookup and a weighted sum of the personalised links).  Wv may be NULL.  Out: O[B][C][d].
 * Chaining the two equals lime_score_candidates up to the storage rounding of W.
 *   lime_score_candidates_gathered:  the same online stage when the cache is one table for the whole item corpus,
 *     Wtable[n_items][h][m] (lime_build_qk_cache with B = 1 and T = the corpus), and a request names its candidates
 *     by id:  O[b][c][head a] = sum_i Wtable[ids[b][c]][a][i] * (LP[b] Wv)[i][head a].  ids: device int32 [B][C];
 *     an id outside [0, n_items) is checked on the device and gives an all-zero output row.  Workspace size as for
 *     LIME_OP_SCORE_CACHED.
 */
int32_t lime_build_qk_cache(const void* T, const void* L, const void* Wq, const void* Wk, void* W,
                            int32_t B, int32_t C, int32_t d, int32_t h, int32_t m,
                            float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream);
int32_t lime_score_candidates_cached(const void* W, const void* LP, const void* Wv, void* O,
                                     int32_t B, int32_t C, int32_t d, int32_t h, int32_t m,
                                     int32_t dtype, void* workspace, size_t ws_bytes, void* stream);
int32_t lime_score_candidates_gathered(const void* Wtable, const int32_t* ids, int32_t n_items, const void* LP,
                                       const void* Wv, void* O, int32_t B, int32_t C, int32_t d, int32_t h, int32_t m,
                                       int32_t dtype, void* workspace, size_t ws_bytes, void* stream);

/*
 * Operands prepared once per model (Section 3.3: what does not depend on the user can be computed ahead of time).
 * Every call above transposes the weights and projects the m links again; with static weights and shared links
 * that work is the same for every request.  lime_prepare does it once into `prepared`, a device buffer of
 * lime_prepared_bytes(d, h, m, dtype) bytes owned by the caller, 256-byte aligned, which holds: for the history
 * stage the W_K^T / W_V images and Q~ = LC Wq_hist (signed by scale_hist); for the candidate stage the W_Q^T image
 * and K~ = L Wk_cand (signed by scale_cand) or, when m <= d/h, their product per head G_a = Wq_cand,a K~_a^T
 * (d x m: the logits of head a are T G_a, one contraction instead of two).  Wq_cand and Wk_cand may be NULL
 * (identity).
 *   lime_link_history_prepared      = lime_link_history (xor_attention = 0) or the LP output of lime_xor_history
 *                                     (xor_attention != 0) with shared links LC[m][d];
 *   lime_score_candidates_prepared  = lime_score_candidates;
 * bit for bit, when given the scale passed to lime_prepare for that stage (only |scale| is read here), except
 * that with m <= d/h the candidate stage rounds G instead of the projected queries to bf16: its outputs then agree
 * with lime_score_candidates within the bf16 tolerance, not bit for bit.  Wv of the
 * candidate stage is still applied per request (the values are the user's link states).  bf16 matrix-core
 * shapes only (see Limits); anything else: lime_prepared_bytes returns 0 and the calls return LIME_UNSUPPORTED.
 * Workspace sizes as for LIME_OP_LINK_HISTORY and LIME_OP_SCORE_CANDIDATES.
 */
size_t lime_prepared_bytes(int32_t d, int32_t h, int32_t m, int32_t dtype);
int32_t lime_prepare(const void* LC, const void* L, const void* Wq_hist, const void* Wk_hist, const void* Wv_hist,
                     const void* Wq_cand, const void* Wk_cand, float scale_hist, float scale_cand,
                     void* prepared, size_t prepared_bytes, int32_t d, int32_t h, int32_t m, int32_t dtype, void* stream);
int32_t lime_link_history_prepared(const void* E, const int32_t* lens, const void* prepared, void* LP,
                                   int32_t B, int32_t N, int32_t d, int32_t h, int32_t m, float scale,
                                   int32_t xor_attention, int32_t dtype, void* workspace, size_t ws_bytes, void* stream);
int32_t lime_score_candidates_prepared(const void* T, const void* LP, const void* Wv, const void* prepared, void* O,
                                       int32_t B, int32_t C, int32_t d, int32_t h, int32_t m, float scale,
                                       int32_t dtype, void* workspace, size_t ws_bytes, void* stream);

/*
 * One request on prepared operands in one call: lime_link_history_prepared followed by lime_score_candidates_prepared
 * (same arguments, same meaning; LP[B][m][d] and O[B][C][d] are both written), as three kernels instead of four: the
 * step that finishes the link states also projects them with the candidate stage's Wv (NULL = identity) into the
 * layout the candidate kernel loads, so the candidate stage packs nothing.  LP is bit-identical to
 * lime_link_history_prepared; O agrees with the two-call form within the bf16 tolerance (the value projection sums
 * in another order).  Workspace: LIME_OP_REQUEST_PREPARED.  Same limits as the other prepared entry points.
 */
int32_t lime_request_prepared(const void* E, const int32_t* lens, const void* T, const void* Wv, const void* prepared,
                              void* LP, void* O, int32_t B, int32_t N, int32_t C, int32_t d, int32_t h, int32_t m,
                              float scale_hist, float scale_cand, int32_t xor_attention, int32_t dtype,
                              void* workspace, size_t ws_bytes, void* stream);

/*
 * One request in one call (Eq. 3 then Eq. 4, or Eq. 7 then Eq. 4): lime_link_history (xor_attention = 0) or the LP
 * output of lime_xor_history (xor_attention != 0) with the *_hist weights and scale_hist, followed by
 * lime_score_candidates on that LP with the *_cand weights and scale_cand.  Arguments, layouts, nullable pointers
 * (Wq_cand, Wk_cand, Wv_cand: NULL = identity) and errors as for those two entry points; LP[B][m][d] and
 * O[B][C][d] are both written, nothing is kept between calls.  On the bf16 matrix-core shapes with 16-byte aligned
 * pointers this is four kernels instead of six: one launch packs the operands of both stages, and the step that
 * finishes the link states also projects them with Wv_cand into the layout the candidate kernel loads.  LP is then
 * bit-identical to lime_link_history / lime_xor_history; O agrees with lime_score_candidates within the bf16
 * tolerance (the value projection sums in another order).  Otherwise the two stages run one after the other as
 * they are.  Workspace: LIME_OP_REQUEST.
 */
int32_t lime_request(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride, const void* Wq_hist,
                     const void* Wk_hist, const void* Wv_hist, const void* T, const void* L, const void* Wq_cand,
                     const void* Wk_cand, const void* Wv_cand, void* LP, void* O, int32_t B, int32_t N, int32_t C,
                     int32_t d, int32_t h, int32_t m, float scale_hist, float scale_cand, int32_t xor_attention,
                     int32_t dtype, void* workspace, size_t ws_bytes, void* stream);

/*
 * lime_request for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and the same bits as lime_request, without the workspace: the
 * scratch memory is a fixed array inside the library's device code (lime_request_static_capacity() bytes, 16 MiB, on
 * every GPU the library runs on, held until the process ends).  The call allocates and frees nothing and calls no
 * allocating routine; its first call on a device looks the array's address up (a host-side query, best made once
 * before any graph capture).  A shape whose kernels need more scratch than the array holds is rejected with
 * LIME_UNSUPPORTED and a message that names both sizes (nothing is enqueued); the headline request (B = 1, N = 2048,
 * C = 32768, d = 256, h = 4, m = 64, bf16) needs 2.7 MiB.  All calls on one GPU share that GPU's array and nothing
 * in it needs clearing between calls (every kernel writes what it later reads), so calls on one GPU must not
 * overlap: two of them in flight at once, on different streams or from different threads, race on the scratch.
 * Calls in order on one stream are safe.
 */
int32_t lime_request_static(const void* E, const int32_t* lens, const void* LC, int64_t lc_user_stride,
                            const void* Wq_hist, const void* Wk_hist, const void* Wv_hist, const void* T, const void* L,
                            const void* Wq_cand, const void* Wk_cand, const void* Wv_cand, void* LP, void* O, int32_t B,
                            int32_t N, int32_t C, int32_t d, int32_t h, int32_t m, float scale_hist, float scale_cand,
                            int32_t xor_attention, int32_t dtype, void* stream);
size_t lime_request_static_capacity(void);

/*
 * Several independent requests (Eq. 3-4 each, Section 3.3: requests of different users share nothing) handed over
 * at once: request i is lime_request(requests[i]...) on streams[i % n_streams].  The requests of one stream are
 * submitted in order by one host thread, those of different streams by different threads (the caller's own for
 * stream 0, threads the library keeps for the others, created on first use and alive until the process ends): a
 * request is four kernel launches, each a few microseconds of host time, and a burst handed over from one thread
 * reaches the GPU that much later.  Every request needs a workspace and an LP of its own (requests in flight at the
 * same time must not share them); the fields are lime_request's arguments with the same meaning, layouts and errors.
 * Returns when everything is enqueued (it does not wait for the GPU); on an error the first failing request's status,
 * with its message in lime_last_error of the calling thread; requests after it on its stream are not submitted, the
 * others may be.  Calls from several threads at once are served one after the other.
 */
typedef struct lime_request_args {
  const void* E; const int32_t* lens; const void* LC; int64_t lc_user_stride;
  const void *Wq_hist, *Wk_hist, *Wv_hist;
  const void *T, *L, *Wq_cand, *Wk_cand, *Wv_cand;
  void *LP, *O;
  int32_t B, N, C, d, h, m;
  float scale_hist, scale_cand;
  int32_t xor_attention, dtype;
  void* workspace; size_t ws_bytes;
} lime_request_args;
int32_t lime_request_many(const lime_request_args* requests, int32_t n, void* const* streams, int32_t n_streams);

/*
 * Backward pass of one XORA layer with respect to its projected inputs (Appendix H.2; forward: Appendix H.1, Eq. 7).
 * Per user b and head (d cut into h contiguous blocks), with S the history rows (lens[b] valid, lens NULL = all N),
 * T the m links and phi(x) = SiLU(scale x) / n:
 *     O[T] = phi(Q[T] K[S]^T) V[S]  (n = lens[b]),        O[S] = phi(Q[S] K[T]^T) V[T]  (n = m).
 * Given the upstream gradients dOT[B][m][d] and dOS[B][N][d] (dOS NULL: O[S] has no consumer, its three gradients
 * are zero) the call writes dQS, dKS, dVS [B][N][d] and dQT, dKT, dVT [B][m][d] (links per user; for shared links
 * the caller sums over users).  For O = phi(Q K^T) V and G = dL/dO:  dV = phi(Z)^T G,  E = (G V^T) * phi'(Z)
 * element-wise,  dQ = scale E K,  dK = scale E^T Q,  Z = scale Q K^T,  SiLU'(x) = s (1 + x (1 - s)), s = sigmoid(x).
 * History rows at or past lens[b] are never read and get zero gradients; a user with lens[b] = 0 gets all zeros.
 * All pointers device memory, row-major, storage type `dtype`; the attention matrices are recomputed in tiles,
 * nothing of size N x m is stored.  bf16 storage with d/h = 32 or 64 and 16-byte aligned pointers runs on the matrix
 * cores (bf16 operands, fp32 accumulation; phi and phi' terms rounded to bf16 before the gradient products), anything
 * else in fp32 arithmetic on the vector ALUs.  Deterministic (no atomics).  d/h <= 64, otherwise LIME_UNSUPPORTED.  Workspace: LIME_OP_XOR_BACKWARD (partial sums of the link-side gradients).
 */
int32_t lime_xor_backward(const void* QS, const void* KS, const void* VS, const void* QT, const void* KT, const void* VT,
                          const void* dOT, const void* dOS, const int32_t* lens, void* dQS, void* dKS, void* dVS,
                          void* dQT, void* dKT, void* dVT, int32_t B, int32_t N, int32_t m, int32_t d, int32_t h,
                          float scale, int32_t dtype, void* workspace, size_t ws_bytes, void* stream);

/*
 * The scoring pipeline around the two attention stages.  The paper names these parts and gives their sizes without
 * defining them; the readings taken here are stated with each.
 *
 * lime_layer_norm - Appendix C ("Model Design", Normalization: layer normalisation before each linear projection in
 *   the QKV projections).  Y[r] = (X[r] - mean) / sqrt(var + eps) * gamma + beta over the d features of row r, biased
 *   variance, statistics in fp32; gamma, beta [d] device pointers in `dtype`, NULL = 1 / 0.  X, Y [rows][d]; Y may be X.
 * lime_contextualize_links - Section 3.1 Eq. 2, L^C = MLP(L (+) E^C): every raw link row L[i] ([m][d], shared) is
 *   concatenated with user b's context vector EC[b] ([B][dc]) and sent through the MLP, read as
 *   ReLU(x W1 + b1) W2 + b2 with W1 [d + dc][dhid], b1 [dhid], W2 [dhid][d], b2 [d] (b1, b2 nullable = 0).
 *   Out: LC[B][m][d] (use it with lc_user_stride = m*d).  Workspace: B * m * dhid floats, rounded up to 256 bytes.
 * lime_interaction_mlp - Section 3.3 (the shallow interaction network; widths as in Appendix C's hyper-parameter
 *   table, e.g. 512, 128, 64): n_maps affine maps x <- x W[i] + b[i], ReLU after all but the last, the last to ONE
 *   logit per row.  W, b, widths are HOST arrays of n_maps entries (device pointers W[i] [d_in][widths[i]] and b[i]
 *   [widths[i]], nullable; widths[n_maps-1] = 1; n_maps <= 4).  In: O[rows][d].  Out: scores[rows], always fp32.
 *   bf16 with (d; hidden widths) in {32, 64, 128, 256} x {(512,128,64), (512,256,128), (96)} (not d = 64 with the
 *   second) runs on the matrix cores with the hidden activations kept in registers (rounded to bf16 between layers);
 *   everything else in fp32 arithmetic.  Workspace: lime_interaction_mlp_workspace_bytes.
 * lime_scores - one LIME-MHA request from embeddings to scores:
 *     L^C = MLP(L (+) E^C)                                   Eq. 2
 *     L^P = MHA(LN(L^C), LN(E), LN(E); theta_hist)           Eq. 3 on normalised inputs, softmax over valid history rows
 *     O   = MHA(LN(T), LN(L), LN(L^P); theta_cand)           Eq. 4 on normalised inputs (keys: raw links, values: L^P)
 *     scores = InteractionMLP(O)                             Section 3.3
 *   Reading of Appendix C's normalisation: every tensor that enters an MHA is layer-normalised once per role - query,
 *   key and value side each with its own (gamma, beta) - and where keys and values are the same tensor (the history
 *   in Eq. 3) one normalisation serves both.  `model` is a HOST struct of device pointers and sizes; E[B][N][d], lens,
 *   EC[B][dc], T[B][C][d] as elsewhere.  Out: scores[B][C] fp32; LC, LP [B][m][d] and O [B][C][d] when not NULL.
 *   Workspace: lime_scores_workspace_bytes, 256-byte aligned (sized for normalised copies of E and T).  For bf16 on the
 *   shapes the matrix-core kernels take, with 16-byte aligned pointers and scale and shift given for every
 *   normalisation, only E is normalised by a pass of its own: L^C, L, L^P and T are normalised inside the kernels that
 *   read them, each rounded to bf16 where the separate pass would have stored it.
 */
typedef struct lime_scoring_model {
  int32_t d, h, m, dc, dhid;  /* embedding width, heads, links, width of the context vector, hidden width of Eq. 2's MLP */
  const void* L;              /* [m][d] raw links */
  const void *ctx_W1, *ctx_b1, *ctx_W2, *ctx_b2;
  const void *hist_Wq, *hist_Wk, *hist_Wv;  /* theta of Eq. 3 */
  const void *cand_Wq, *cand_Wk, *cand_Wv;  /* theta of Eq. 4 (all three required here) */
  const void* ln_hist_q[2];   /* (gamma, beta) of the layer normalisation of L^C; each [d], NULL = 1 / 0 */
  const void* ln_hist_kv[2];  /* of E (keys and values of Eq. 3) */
  const void* ln_cand_q[2];   /* of T */
  const void* ln_cand_k[2];   /* of L */
  const void* ln_cand_v[2];   /* of L^P */
  int32_t n_mlp;              /* affine maps of the interaction network (1..4), the last to one logit */
  int32_t mlp_width[4];
  const void* mlp_W[4];
  const void* mlp_b[4];
  float scale_hist, scale_cand, ln_eps;
} lime_scoring_model;

int32_t lime_layer_norm(const void* X, const void* gamma, const void* beta, float eps, void* Y, int64_t rows, int32_t d,
                        int32_t dtype, void* stream);
int32_t lime_contextualize_links(const void* L, const void* EC, const void* W1, const void* b1, const void* W2, const void* b2,
                                 void* LC, int32_t B, int32_t m, int32_t d, int32_t dc, int32_t dhid, int32_t dtype,
                                 void* workspace, size_t ws_bytes, void* stream);
size_t lime_interaction_mlp_workspace_bytes(int64_t rows, int32_t d, const int32_t* widths, int32_t n_maps, int32_t dtype);
int32_t lime_interaction_mlp(const void* O, const void* const* W, const void* const* b, const int32_t* widths, int32_t n_maps,
                             float* scores, int64_t rows, int32_t d, int32_t dtype, void* workspace, size_t ws_bytes, void* stream);
size_t lime_scores_workspace_bytes(const lime_scoring_model* model, int32_t B, int32_t N, int32_t C, int32_t dtype);
int32_t lime_scores(const lime_scoring_model* model, const void* E, const int32_t* lens, const void* EC, const void* T,
                    void* LC, void* LP, void* O, float* scores, int32_t B, int32_t N, int32_t C, int32_t dtype,
                    void* workspace, size_t ws_bytes, void* stream);

/*
 * Workspace size in bytes for `op` (LIME_OP_*) at the given shape; dimensions an op
 * does not have are ignored.  `flags` bit 0: lime_xor_history will be asked for OS.
 * Returns 0 for shapes the op would reject.
 */
size_t lime_workspace_bytes(int32_t op, int32_t B, int32_t N, int32_t C, int32_t d, int32_t h, int32_t m,
                            int32_t dtype, int32_t flags);

/*
 * Per-kernel timing for benchmarks (callers that only want results never need it; these are the only functions of
 * the library that create HIP events and wait on the device).
 * lime_profile_enable(1): from now on every main kernel launched by the entry points above carries a start and a
 * stop event of its own (hipExtLaunchKernel), which the runtime fills with the dispatch's begin and end time stamps:
 * the kernel's own duration as a kernel trace reports it.  Kernel ids: 0 = the candidate-side kernel of
 * lime_score_candidates and of O[S]; 1 = the links-over-history kernel of lime_link_history / lime_xor_history;
 * 2 = the attention kernel of mha_target_attention; 3 = its three row projections (one duration each); 4 = the kernel
 * of lime_score_candidates_cached and lime_score_candidates_gathered; 5, 6 = the two probes below.
 * lime_profile_collect(kernel, ms, capacity): waits for the recorded launches of that kernel,
 * writes up to `capacity` durations in milliseconds to the HOST array `ms` in launch order,
 * forgets them and returns how many it wrote.  Only the matrix-core kernels are instrumented.
 */
void lime_profile_enable(int32_t on);
int32_t lime_profile_collect(int32_t kernel, float* ms, int32_t capacity);

/*
 * Achievable-peak probes for the benchmark's roofline context (Section 4 "Inference Speed" is measured against a
 * machine; these say what this one sustains).  lime_probe_copy: a plain streaming copy of `bytes` (a multiple of 16,
 * both pointers 16-byte aligned device memory) on `stream`; returns a status.  lime_probe_mfma: every compute unit
 * runs `iters` x 4 register-resident v_mfma_f32_32x32x16_bf16 per wave; `out` is device memory of
 * lime_probe_mfma_out_bytes() bytes; returns the floating-point operations the launch executes (0 on error).
 * Time either with lime_profile_enable / lime_profile_collect (kernel ids 5 and 6).
 */
int32_t lime_probe_copy(const void* src, void* dst, size_t bytes, void* stream);
size_t lime_probe_mfma_out_bytes(void);
double lime_probe_mfma(void* out, int32_t iters, void* stream);

/* Text of the calling thread's most recent non-zero status ("" if none).  Host memory, owned by the library. */
const char* lime_last_error(void);

/* "major.minor.patch" of the library.  Host memory, owned by the library. */
const char* lime_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LIME_H_ */
